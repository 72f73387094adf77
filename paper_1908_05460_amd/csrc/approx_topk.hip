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

__device__ __forceinline__ unsigned long long wave_max(unsigned long long v)
{
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const unsigned long long o = __shfl_xor(v, d, 64);
        v = o > v ? o : v;
    }
    return v;
}

// One wavefront per map (WIDE = false), or one workgroup per map for maps of more than 1024 positions
// (WIDE = true: few, long maps would otherwise leave most of the chip idle).  Pass j finds the largest key
// below the one pass j-1 found, so no list of taken positions is kept; the map's sum rides along with pass 0.
// Maps of up to T*REG entries (T = 64 or 256 threads) stay in registers between the passes, longer ones are
// read again (from L2).
template <bool BF16, int REG, bool WIDE>
__global__ __launch_bounds__(kBlock) void topk_select(const void *__restrict__ dY, long maps, int len, int Wo,
                                                      int k, int32_t *__restrict__ hw_out,
                                                      int32_t *__restrict__ flat_out, float *__restrict__ sum_a,
                                                      float *__restrict__ sum_b)
{
    constexpr int T = WIDE ? kBlock : 64;
    __shared__ unsigned long long wg_best[2][kBlock / 64];      // WIDE: the wavefronts' maxima, double-buffered over passes
    __shared__ float wg_sum[kBlock / 64];
    const int lane = WIDE ? threadIdx.x : threadIdx.x & 63;
    const long map = WIDE ? (long)blockIdx.x : (long)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (map >= maps) return;                      // whole wavefronts leave together (WIDE: the grid is exactly maps)
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
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) sum += __shfl_xor(sum, d, 64);
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
        best = wave_max(best);
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
    return align_up(maps * k * sizeof(int32_t)) + align_up(maps * sizeof(float)) + topk_partial_bytes(g);
}

int launch_approx_topk(const Geometry &g, const void *X, const void *dY, float *dW, int k, float scale,
                       int32_t *idx_out, float *sum_out, void *ws, hipStream_t st)
{
    const long maps = (long)g.N * g.K;
    const int len = g.Ho * g.Wo;
    char *w = (char *)ws;
    int32_t *hw = (int32_t *)w;  w += align_up((size_t)maps * k * sizeof(int32_t));
    float *sum = (float *)w;     w += align_up((size_t)maps * sizeof(float));
    float *partials = (float *)w;

    int rc;
    // maps of up to 1024 positions and C*R*S <= 576: selection and gather in one launch
    if (topk_fused(g, X, dY, k, scale, dW, idx_out, sum_out, partials, st, &rc)) return rc;

    const bool wide = len > 1024;
    const long grid = wide ? maps : (maps + kBlock / 64 - 1) / (kBlock / 64);
    if (grid >= (1l << 31)) return WGRAD_UNSUPPORTED;
#define SEL_ARGS dim3((unsigned)grid), dim3(kBlock), 0, st, dY, maps, len, g.Wo, k, hw, idx_out, sum, sum_out
#define SEL_PICK(BF)                                                                     \
    if (len <= 64)        WGRAD_LAUNCH((topk_select<BF, 1, false>), SEL_ARGS);           \
    else if (len <= 256)  WGRAD_LAUNCH((topk_select<BF, 4, false>), SEL_ARGS);           \
    else if (len <= 1024) WGRAD_LAUNCH((topk_select<BF, 16, false>), SEL_ARGS);          \
    else if (len <= 4096) WGRAD_LAUNCH((topk_select<BF, 16, true>), SEL_ARGS);           \
    else                  WGRAD_LAUNCH((topk_select<BF, 0, true>), SEL_ARGS)
    if (g.bf16) { SEL_PICK(true); } else { SEL_PICK(false); }
#undef SEL_PICK
#undef SEL_ARGS
    rc = launch_status();
    if (rc != WGRAD_OK) return rc;

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
