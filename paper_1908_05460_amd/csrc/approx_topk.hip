// Top-k generalisation of the max-gradient approximation (arXiv 1908.05460, Section 2.3):
// every map of dY keeps its k entries of largest magnitude instead of one, and each kept
// position carries sum/k, so that the k = 1 case is Algorithm 1 and the retained mass is
// the map's sum whatever k is.  Two kernels: selection, then a gather over the kept
// positions; the batch-chunk partials go through the common reduction.
#include "common.hpp"

namespace wgrad {

namespace {

// A position's rank key: magnitude bits above, inverted index below.  Keys of one map are
// all different, and "larger magnitude first, smaller index first among equals" is plain
// descending key order.  NaN ranks as zero magnitude.
__device__ __forceinline__ unsigned long long rank_key(uint32_t bits, uint32_t pos)
{
    uint32_t m = bits & 0x7fffffffu;
    m = m > 0x7f800000u ? 0u : m;
    return ((unsigned long long)m << 32) | (uint32_t)~pos;
}

template <bool BF16>
__device__ __forceinline__ uint32_t load_bits(const void *p, long i)
{
    return BF16 ? (uint32_t)((const uint16_t *)p)[i] << 16 : ((const uint32_t *)p)[i];
}

// maximum over aligned groups of G lanes (G a power of two up to 64)
__device__ __forceinline__ unsigned long long group_max(unsigned long long v, int G)
{
    for (int d = G >> 1; d > 0; d >>= 1) {
        const unsigned long long o = __shfl_xor(v, d, 64);
        v = o > v ? o : v;
    }
    return v;
}

// A group of G lanes per map (WIDE = false; G a power of two, 64 / G maps per wavefront, so that maps of four
// positions take a lane each and not a wavefront each), or one workgroup per map for maps of more than 1024
// positions (WIDE = true: few, long maps would otherwise leave most of the chip idle).  Pass j finds the largest
// key below the one pass j-1 found, so no list of taken positions is kept; the map's sum rides along with pass 0.
// Maps of up to T*REG entries (T = G or 256 threads) stay in registers between the passes, longer ones are
// read again (from L2).
template <bool BF16, int REG, bool WIDE>
__global__ __launch_bounds__(kBlock) void topk_select(const void *__restrict__ dY, long maps, int len, int Wo,
                                                      int k, int G, int32_t *__restrict__ hw_out,
                                                      int32_t *__restrict__ flat_out, float *__restrict__ sum_a,
                                                      float *__restrict__ sum_b, void *__restrict__ sparse, float w)
{
    const int T = WIDE ? kBlock : G;
    __shared__ unsigned long long wg_best[2][kBlock / 64];      // WIDE: the wavefronts' maxima, double-buffered over passes
    __shared__ float wg_sum[kBlock / 64];
    const int lane = WIDE ? threadIdx.x : (threadIdx.x & 63) % G;
    const long map = WIDE ? (long)blockIdx.x
                          : ((long)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)) * (64 / G) + (threadIdx.x & 63) / G;
    if (map >= maps) return;                      // whole groups leave together (WIDE: the grid is exactly maps)
    const long base = map * len;

    unsigned long long held[REG > 0 ? REG : 1];
    float sum = 0.f;
    if (REG > 0) {
#pragma unroll
        for (int i = 0; i < REG; ++i) {
            const int e = lane + T * i;
            held[i] = 0ull;                        // below every real key: ~pos is never 0 for pos < 2^32-1
            if (e < len) {
                const uint32_t b = load_bits<BF16>(dY, base + e);
                held[i] = rank_key(b, (uint32_t)e);
                sum += __uint_as_float(b);
            }
        }
    } else {
        for (int e = lane; e < len; e += T) sum += __uint_as_float(load_bits<BF16>(dY, base + e));
    }
    for (int d = (WIDE ? 64 : G) >> 1; d > 0; d >>= 1) sum += __shfl_xor(sum, d, 64);
    if (WIDE) {
        if ((threadIdx.x & 63) == 0) wg_sum[threadIdx.x >> 6] = sum;
        __syncthreads();
        sum = (wg_sum[0] + wg_sum[1]) + (wg_sum[2] + wg_sum[3]);
    }

    unsigned long long below = ~0ull;
    for (int j = 0; j < k; ++j) {
        unsigned long long best = 0ull;
        if (REG > 0) {
#pragma unroll
            for (int i = 0; i < REG; ++i) {
                const unsigned long long c = held[i] < below ? held[i] : 0ull;
                best = c > best ? c : best;
            }
        } else {
            for (int e = lane; e < len; e += T) {
                unsigned long long c = rank_key(load_bits<BF16>(dY, base + e), (uint32_t)e);
                c = c < below ? c : 0ull;
                best = c > best ? c : best;
            }
        }
        best = group_max(best, WIDE ? 64 : G);
        if (WIDE) {
            // pass j writes buffer j & 1; the barrier of pass j+1 separates its readers from pass j+2's writers
            if ((threadIdx.x & 63) == 0) wg_best[j & 1][threadIdx.x >> 6] = best;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < kBlock / 64; ++w) best = wg_best[j & 1][w] > best ? wg_best[j & 1][w] : best;
        }
        below = best;
        if (threadIdx.x == 0 || (!WIDE && lane == 0)) {
            const int32_t pos = (int32_t)~(uint32_t)best;
            if (flat_out) flat_out[map * k + j] = pos;
            hw_out[map * k + j] = ((pos / Wo) << 16) | (pos % Wo);
        }
    }
    if (threadIdx.x == 0 || (!WIDE && lane == 0)) {
        sum_a[map] = sum;
        if (sum_b) sum_b[map] = sum;
    }
    // optional: the sparsified map, sum * w at the kept positions (the k largest keys: those not below the
    // last one found) and zero elsewhere, in the element type of the inputs
    if (sparse) {
        const float kept = sum * w;
        auto put = [&](int e, bool is_kept) {
            const float v = is_kept ? kept : 0.f;
            if (BF16) {
                const uint32_t b = __float_as_uint(v);           // round to nearest even; v is finite
                ((uint16_t *)sparse)[base + e] = (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
            } else {
                ((float *)sparse)[base + e] = v;
            }
        };
        if (REG > 0) {
#pragma unroll
            for (int i = 0; i < REG; ++i) {
                const int e = lane + T * i;
                if (e < len) put(e, held[i] >= below);
            }
        } else {
            for (int e = lane; e < len; e += T)
                put(e, rank_key(load_bits<BF16>(dY, base + e), (uint32_t)e) >= below);
        }
    }
}

// One thread per filter-gradient entry (ko, c, r, s) and batch chunk: it walks the chunk's
// images and the k kept positions of map (n, ko), adding (sum/k) times the input element
// its tap sees there (zero outside the image).
template <bool BF16>
__global__ __launch_bounds__(kBlock) void topk_gather(const void *__restrict__ X, const int32_t *__restrict__ hw,
                                                      const float *__restrict__ sum, float *__restrict__ out,
                                                      Geometry g, int k, float inv_k, int chunk_n, float scale)
{
    const long o = (long)blockIdx.x * kBlock + threadIdx.x;
    const int RS = g.R * g.S, CRS = g.C * RS;
    if (o >= (long)g.K * CRS) return;
    const int ko = (int)(o / CRS), q = (int)(o % CRS);
    const int c = q / RS, r = (q % RS) / g.S, s = q % g.S;
    const int n_begin = blockIdx.y * chunk_n;
    const int n_end = n_begin + chunk_n < g.N ? n_begin + chunk_n : g.N;
    float acc = 0.f;
    for (int n = n_begin; n < n_end; ++n) {
        const long m = (long)n * g.K + ko;
        const float share = sum[m] * inv_k;
        const long plane = ((long)n * g.C + c) * g.H;
        float part = 0.f;
#pragma unroll 4
        for (int j = 0; j < k; ++j) {
            const int p = hw[m * k + j];
            const int ih = (p >> 16) * g.sh + r - g.ph, iw = (p & 0xffff) * g.sw + s - g.pw;
            if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
                const long xi = (plane + ih) * g.W + iw;
                part += BF16 ? bf16_bits_to_float(((const uint16_t *)X)[xi]) : ((const float *)X)[xi];
            }
        }
        acc = fmaf(share, part, acc);
    }
    out[(long)blockIdx.y * g.K * CRS + o] = acc * scale;
}

// When the kept positions are a sizeable share of a map, gathering their patches moves as much data as the
// dense kernel and loses to the matrix core: the gradient is then computed as the exact gradient of the
// sparsified dY (Section 2.4's identity).  Thresholds from measurements on the VGG-19 layers (N = 128): the
// LDS gather costs about k/2 of the dense kernel on 4x4 planes and k/5 on 8x8 planes; the general gather
// loses from three kept positions of 256 on; with bf16 inputs the dense kernel is twice as fast again.
bool topk_sparse_exact(const Geometry &g, int k, ExactPlan &ex)
{
    if (!tune_int("WGRAD_TOPK_SX", 1)) return false;
    const int L = g.Ho * g.Wo;
    ex = plan_exact(g);
    if (!ex.ok) return false;
    // the bf16 matrix-core kernel runs a dense layer in the time the gather needs for one kept position
    const bool fast_bf16 = ex.mm16 && k >= 2;
    // large maps, few channels: the fused kernel, unless the bf16 matrix core beats it (maps of up to 256 positions)
    if (topk_takes_fused(g, k)) return fast_bf16 && L <= 256;
    const ApproxPlan ap = plan_approx(g, /*allow_lds=*/true, /*allow_fused=*/false, /*allow_mm=*/false);
    const bool lds = ap.use_lds && ap.m * k <= 64;
    const bool dense_enough = L <= 4 || (lds ? k >= 2 && k * 14 >= L : k * 80 >= L);
    return fast_bf16 || ((ex.stream || ex.mm16) && dense_enough);
}

int topk_chunks(const Geometry &g)
{
    // enough (entry, chunk) threads to fill the chip, at least 4 images per chunk
    const long entries = g.dw_elems();
    long chunks = (256l * 1024 + entries - 1) / entries;
    const long most = (g.N + 3) / 4;
    chunks = chunks > most ? most : chunks;
    return (int)(chunks < 1 ? 1 : chunks);
}

}  // namespace

bool topk_supported(const Geometry &g, int k)
{
    return k >= 1 && k <= kTopKMax && (long)k <= (long)g.Ho * g.Wo && g.Ho < 32768 && g.Wo < 65536;
}

// batch-chunk partials of whichever form runs: the general gather here, the fused kernel or the LDS gather
static size_t topk_partial_bytes(const Geometry &g)
{
    const int chunks = topk_chunks(g);
    size_t general = chunks > 1 ? (size_t)chunks * g.dw_elems() * sizeof(float) : 0;
    const size_t borrowed = topk_borrowed_partial_bytes(g);
    return align_up(general > borrowed ? general : borrowed);
}

size_t topk_ws_bytes(const Geometry &g, int k)
{
    const size_t maps = (size_t)g.N * g.K;
    size_t tail = topk_partial_bytes(g);
    ExactPlan ex;
    if (topk_sparse_exact(g, k, ex)) {
        const size_t sx = align_up(maps * g.Ho * g.Wo * (g.bf16 ? 2 : 4)) + align_up(ex.ws_bytes);
        if (sx > tail) tail = sx;
    }
    return align_up(maps * k * sizeof(int32_t)) + align_up(maps * sizeof(float)) + tail;
}

bool launch_topk_group(const Geometry &g, const Batch &b, int k, float scale, void *ws, size_t slice_bytes,
                       hipStream_t st, int *rc, FusedQueue *fq, CombineQueue *defer)
{
    ExactPlan ex;
    if (topk_sparse_exact(g, k, ex)) return false;         // that form runs layer by layer
    // a slice holds the kept positions, the sums, then the partials (as in launch_approx_topk)
    const long maps = (long)g.N * g.K;
    const size_t off = align_up((size_t)maps * k * sizeof(int32_t)) + align_up((size_t)maps * sizeof(float));
    return topk_fused(g, b, k, scale, nullptr, nullptr, (float *)((char *)ws + off), (long)(slice_bytes / 4), st, rc, fq, defer);
}

// fq, defer: a schedule run's queue of fused launches and of reductions (the fused form then only records its work)
int launch_approx_topk(const Geometry &g, const void *X, const void *dY, float *dW, int k, float scale,
                       int32_t *idx_out, float *sum_out, void *ws, hipStream_t st, FusedQueue *fq, CombineQueue *defer)
{
    const long maps = (long)g.N * g.K;
    const int len = g.Ho * g.Wo;
    char *w = (char *)ws;
    int32_t *hw = (int32_t *)w;  w += align_up((size_t)maps * k * sizeof(int32_t));
    float *sum = (float *)w;     w += align_up((size_t)maps * sizeof(float));
    float *partials = (float *)w;

    int rc;
    // kept positions a sizeable share of a map: the selection also writes the sparsified dY, and the exact
    // kernel contracts it
    ExactPlan ex;
    const bool sx = topk_sparse_exact(g, k, ex);
    void *sparse = sx ? (void *)partials : nullptr;
    // maps of up to 1024 positions and C*R*S <= 2304: selection and gather in one launch
    Batch one{};
    one.n = 1; one.X[0] = X; one.dY[0] = dY; one.dW[0] = dW;
    if (!sx && topk_fused(g, one, k, scale, idx_out, sum_out, partials, 0, st, &rc, fq, defer)) return rc;

    const bool wide = len > 1024;
    // lanes per map: four positions each up to 256 positions, sixteen up to 1024
    int G = 1;
    while (G < 64 && G * 4 < len) G <<= 1;
    const long waves = (maps + 64 / G - 1) / (64 / G);
    const long grid = wide ? maps : (waves + kBlock / 64 - 1) / (kBlock / 64);
    if (grid >= (1l << 31)) return WGRAD_UNSUPPORTED;
#define SEL_ARGS dim3((unsigned)grid), dim3(kBlock), 0, st, dY, maps, len, g.Wo, k, G, hw, idx_out, sum, sum_out, sparse, scale / k
#define SEL_PICK(BF)                                                                     \
    if (len <= 256)       WGRAD_LAUNCH((topk_select<BF, 4, false>), SEL_ARGS);           \
    else if (len <= 1024) WGRAD_LAUNCH((topk_select<BF, 16, false>), SEL_ARGS);          \
    else if (len <= 4096) WGRAD_LAUNCH((topk_select<BF, 16, true>), SEL_ARGS);           \
    else                  WGRAD_LAUNCH((topk_select<BF, 0, true>), SEL_ARGS)
    if (g.bf16) { SEL_PICK(true); } else { SEL_PICK(false); }
#undef SEL_PICK
#undef SEL_ARGS
    rc = launch_status();
    if (rc != WGRAD_OK) return rc;

    if (sx) {
        Batch eb{};
        eb.n = 1; eb.X[0] = X; eb.dY[0] = sparse; eb.dW[0] = dW;
        return launch_exact(g, ex, eb, (char *)partials + align_up((size_t)maps * len * (g.bf16 ? 2 : 4)), st);
    }

    // small planes and many output channels: the LDS-staged gather of the k = 1 path, over k positions per map
    if (topk_gather_lds(g, X, hw, sum, k, scale, dW, partials, topk_partial_bytes(g), st, &rc)) return rc;

    const int chunks = topk_chunks(g);
    const int chunk_n = (g.N + chunks - 1) / chunks;
    const int nchunk = (g.N + chunk_n - 1) / chunk_n;
    const long entries = g.dw_elems();
    float *out = nchunk > 1 ? partials : dW;
    const dim3 gg((unsigned)((entries + kBlock - 1) / kBlock), (unsigned)nchunk);
    const float gscale = nchunk > 1 ? 1.0f : scale;
    if (g.bf16) WGRAD_LAUNCH((topk_gather<true>), gg, dim3(kBlock), 0, st, X, hw, sum, out, g, k, 1.0f / k, chunk_n, gscale);
    else        WGRAD_LAUNCH((topk_gather<false>), gg, dim3(kBlock), 0, st, X, hw, sum, out, g, k, 1.0f / k, chunk_n, gscale);
    rc = launch_status();
    if (rc != WGRAD_OK || nchunk == 1) return rc;
    float *dst[1] = {dW};
    return launch_combine(partials, 0, nchunk, entries, scale, dst, 1, st, nullptr);
}

}  // namespace wgrad
