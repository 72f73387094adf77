// Max Gradient Approximation (Algorithm 1 of arXiv 1908.05460) on gfx950.
//
//   select :  for every map dY[n,k,:,:]   idx = argmax |dY| (lowest flat position on
//             ties),  S = signed sum of the map                  -- streams dY once
//   gather :  dW[k,c,r,s] = scale * sum_n S[n,k] * X[n,c,h* sh + r - ph, w* sw + s - pw]
//             (zero outside X)                                    -- reads the patches
//   combine:  sums the batch-chunk partials of the gather (shared with the exact path).
#include "common.hpp"

namespace wgrad {

// ------------------------------------------------------------------------------------
// select: a group of G lanes (power of two, <= 64) owns one map; each lane walks the
// map in 16-byte pieces G pieces apart, keeps its own best (|v| bits, position) and
// partial sum, then the group reduces with a butterfly over lane-xor shuffles.
//
// The comparison is done on the magnitude bits as unsigned integers, which orders
// finite floats (and infinities) exactly as |v| does; +0/-0 and +v/-v compare equal.
// A NaN gets key 0 so it can never displace anything, as with a strict '>' on floats.
// Ties go to the lowest position: within a lane positions are visited in ascending
// order with a strict '>', and across lanes the packed key (mag << 32 | ~pos) is
// maximised, which prefers the larger magnitude and then the smaller position.
// ------------------------------------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ uint32_t mag_key(uint32_t bits)   // bits of the value as fp32
{
    const uint32_t m = bits & 0x7fffffffu;
    return m > 0x7f800000u ? 0u : m;
}

template <bool BF16, int VEC>
__global__ __launch_bounds__(kBlock) void approx_select(const void *__restrict__ dY, long maps, int len,
                                                        int G, int32_t *__restrict__ idx_a,
                                                        float *__restrict__ sum_a,
                                                        int32_t *__restrict__ idx_b,
                                                        float *__restrict__ sum_b)
{
    const int lane = threadIdx.x & 63;
    const int maps_per_wave = 64 / G;
    const long wave_global = (long)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    const long map = wave_global * maps_per_wave + lane / G;
    const int gl = lane % G;

    uint32_t best_key = 0, best_pos = 0;
    bool have = false;
    float sum = 0.f;
    if (map < maps) {
        const long base = map * len;
#pragma unroll 4
        for (int e = gl * VEC; e < len; e += G * VEC) {
            uint32_t bits[VEC];
            if (VEC == 1) {
                bits[0] = BF16 ? (uint32_t)((const uint16_t *)dY)[base + e] << 16
                               : ((const uint32_t *)dY)[base + e];
            } else if (BF16) {   // VEC == 8 : one 16-byte load of 8 bf16
                const uint4 raw = *(const uint4 *)((const uint16_t *)dY + base + e);
                const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) { bits[2 * i] = w[i] << 16; bits[2 * i + 1] = w[i] & 0xffff0000u; }
            } else {             // VEC == 4 : one 16-byte load of 4 fp32
                const uint4 raw = *(const uint4 *)((const uint32_t *)dY + base + e);
                bits[0] = raw.x; bits[1] = raw.y; bits[2] = raw.z; bits[3] = raw.w;
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const uint32_t key = mag_key<BF16>(bits[i]);
                if (!have || key > best_key) { best_key = key; best_pos = e + i; have = true; }
                sum += __uint_as_float(bits[i]);
            }
        }
    }
    // lanes that saw nothing (len smaller than the group's reach) must lose every comparison
    unsigned long long packed = have ? ((unsigned long long)best_key << 32) | (uint32_t)~best_pos : 0ull;
    for (int d = G >> 1; d > 0; d >>= 1) {
        const unsigned long long other = __shfl_xor(packed, d, 64);
        const float osum = __shfl_xor(sum, d, 64);
        packed = other > packed ? other : packed;
        sum += osum;
    }
    if (map < maps && gl == 0) {
        const int32_t pos = (int32_t)~(uint32_t)packed;
        idx_a[map] = pos;
        sum_a[map] = sum;
        if (idx_b) idx_b[map] = pos;
        if (sum_b) sum_b[map] = sum;
    }
}

int launch_select2(const Geometry &g, const void *dY, int32_t *idx_a, float *sum_a, int32_t *idx_b,
                   float *sum_b, hipStream_t st)
{
    const int len = g.Ho * g.Wo;
    const long maps = (long)g.N * g.K;
    const int full = g.bf16 ? 8 : 4;                      // elements per 16-byte access
    const bool vec_ok = len % full == 0 && ((uintptr_t)dY % 16) == 0;
    const int vec = vec_ok ? full : 1;
    // lanes per map: enough that each lane issues about four accesses
    int G = 1;
    while (G < 64 && G * vec * 4 < len) G <<= 1;
    const long waves = (maps + 64 / G - 1) / (64 / G);
    const int grid = (int)((waves + kBlock / 64 - 1) / (kBlock / 64));
    if (g.bf16) {
        if (vec == 8) WGRAD_LAUNCH((approx_select<true, 8>), dim3(grid), dim3(kBlock), 0, st, dY, maps, len, G, idx_a, sum_a, idx_b, sum_b);
        else          WGRAD_LAUNCH((approx_select<true, 1>), dim3(grid), dim3(kBlock), 0, st, dY, maps, len, G, idx_a, sum_a, idx_b, sum_b);
    } else {
        if (vec == 4) WGRAD_LAUNCH((approx_select<false, 4>), dim3(grid), dim3(kBlock), 0, st, dY, maps, len, G, idx_a, sum_a, idx_b, sum_b);
        else          WGRAD_LAUNCH((approx_select<false, 1>), dim3(grid), dim3(kBlock), 0, st, dY, maps, len, G, idx_a, sum_a, idx_b, sum_b);
    }
    return launch_status();
}

int launch_select(const Geometry &g, const void *dY, int32_t *idx, float *sum, hipStream_t st)
{
    return launch_select2(g, dY, idx, sum, nullptr, nullptr, st);
}

// ------------------------------------------------------------------------------------
// gather, direct form: one thread per filter-gradient entry (k, c, r, s) and batch
// chunk; it walks the chunk's images, reads the map's (idx, S) and the one input
// element its tap sees.  Used when the patches touch only part of each input plane.
// ------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(kBlock) void approx_gather_direct(const void *__restrict__ X,
                                                               const int32_t *__restrict__ idx,
                                                               const float *__restrict__ sum,
                                                               float *__restrict__ out, Geometry g,
                                                               int chunk_n, float scale)
{
    const long o = (long)blockIdx.x * kBlock + threadIdx.x;
    const int RS = g.R * g.S, CRS = g.C * RS;
    if (o >= (long)g.K * CRS) return;
    const int k = (int)(o / CRS), j = (int)(o % CRS);
    const int c = j / RS, r = (j % RS) / g.S, s = j % g.S;
    const int n_begin = blockIdx.y * chunk_n;
    const int n_end = n_begin + chunk_n < g.N ? n_begin + chunk_n : g.N;
    float acc = 0.f;
#pragma unroll 4
    for (int n = n_begin; n < n_end; ++n) {
        const int pos = idx[(long)n * g.K + k];
        const float sv = sum[(long)n * g.K + k];
        const int ih = (pos / g.Wo) * g.sh + r - g.ph, iw = (pos % g.Wo) * g.sw + s - g.pw;
        if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
            const long xi = (((long)n * g.C + c) * g.H + ih) * g.W + iw;
            const float xv = BF16 ? bf16_bits_to_float(((const uint16_t *)X)[xi]) : ((const float *)X)[xi];
            acc = fmaf(sv, xv, acc);
        }
    }
    out[(long)blockIdx.y * g.K * CRS + o] = acc * scale;
}

#ifndef WGRAD_APPROX_THREADS   // threads to aim for when chunking the batch
#define WGRAD_APPROX_THREADS (256 * 1024)
#endif

ApproxPlan plan_approx(const Geometry &g)
{
    ApproxPlan pl{};
    const long outs = g.dw_elems();
    long chunks = (WGRAD_APPROX_THREADS + outs - 1) / outs;
    if (chunks > g.N) chunks = g.N;
    if (chunks < 1) chunks = 1;
    const int chunk_n = (int)((g.N + chunks - 1) / chunks);
    pl.chunks = (g.N + chunk_n - 1) / chunk_n;
    size_t off = 0;
    pl.off_idx = off; off += align_up((size_t)g.N * g.K * 4);
    pl.off_sum = off; off += align_up((size_t)g.N * g.K * 4);
    pl.off_part = off; off += pl.chunks > 1 ? align_up((size_t)pl.chunks * outs * 4) : 0;
    pl.ws_bytes = off;
    return pl;
}

int launch_approx(const Geometry &g, const ApproxPlan &pl, const void *X, const void *dY, float *dW,
                  float scale, int32_t *idx_out, float *sum_out, void *ws, hipStream_t st)
{
    int32_t *idx = (int32_t *)((char *)ws + pl.off_idx);
    float *sum = (float *)((char *)ws + pl.off_sum);
    float *part = (float *)((char *)ws + pl.off_part);
    int rc = launch_select2(g, dY, idx, sum, idx_out, sum_out, st);
    if (rc != WGRAD_OK) return rc;

    const long outs = g.dw_elems();
    const int chunk_n = (g.N + pl.chunks - 1) / pl.chunks;
    const dim3 grid((unsigned)((outs + kBlock - 1) / kBlock), (unsigned)pl.chunks);
    float *out = pl.chunks > 1 ? part : dW;
    const float kscale = pl.chunks > 1 ? 1.0f : scale;
    if (g.bf16) WGRAD_LAUNCH((approx_gather_direct<true>), grid, dim3(kBlock), 0, st, X, idx, sum, out, g, chunk_n, kscale);
    else        WGRAD_LAUNCH((approx_gather_direct<false>), grid, dim3(kBlock), 0, st, X, idx, sum, out, g, chunk_n, kscale);
    rc = launch_status();
    if (rc != WGRAD_OK) return rc;
    if (pl.chunks > 1) return launch_combine(part, pl.chunks, outs, scale, dW, st);
    return WGRAD_OK;
}

// ------------------------------------------------------------------------------------
// combine: dW[o] = scale * sum_i partial[i][o], summed in ascending i (deterministic).
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void combine_partials(const float *__restrict__ part, int nparts,
                                                           long elems, float scale, float *__restrict__ dW)
{
    const long o = (long)blockIdx.x * kBlock + threadIdx.x;
    if (o >= elems) return;
    float acc = 0.f;
#pragma unroll 8
    for (int i = 0; i < nparts; ++i) acc += part[(long)i * elems + o];
    dW[o] = acc * scale;
}

int launch_combine(const float *partials, int nparts, long elems, float scale, float *dW, hipStream_t st)
{
    const int grid = (int)((elems + kBlock - 1) / kBlock);
    WGRAD_LAUNCH(combine_partials, dim3(grid), dim3(kBlock), 0, st, partials, nparts, elems, scale, dW);
    return launch_status();
}

}  // namespace wgrad
