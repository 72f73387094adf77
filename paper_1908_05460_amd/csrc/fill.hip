// The two trivial gradient methods of arXiv 1908.05460: zero gradient (Section 2.1)
// and random gradient (Section 2.2).
#include "common.hpp"

namespace wgrad {

// A workgroup clears kZeroPerBlock consecutive floats: four 16-byte stores per thread, each store instruction
// of a wavefront covering 1 KB of consecutive addresses (a workgroup per 4 KB spent more time being dispatched
// than storing).
constexpr int kZeroPieces = 4;
constexpr long kZeroPerBlock = (long)kBlock * 4 * kZeroPieces;

__device__ __forceinline__ void zero_block(float *__restrict__ dW, long elems, long block)
{
    const bool aligned = ((uintptr_t)dW % 16) == 0;
#pragma unroll
    for (int p = 0; p < kZeroPieces; ++p) {
        const long i = block * kZeroPerBlock + ((long)p * kBlock + threadIdx.x) * 4;
        if (i + 3 < elems && aligned) {
            *(float4 *)(dW + i) = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            for (long j = i; j < elems && j < i + 4; ++j) dW[j] = 0.f;
        }
    }
}

__global__ __launch_bounds__(kBlock) void fill_zero(float *__restrict__ dW, long elems)
{
    zero_block(dW, elems, blockIdx.x);
}

int launch_zero(float *dW, long elems, hipStream_t st)
{
    const long blocks = (elems + kZeroPerBlock - 1) / kZeroPerBlock;
    if (blocks >= (1l << 31)) return WGRAD_UNSUPPORTED;
    WGRAD_LAUNCH(fill_zero, dim3((unsigned)(blocks < 1 ? 1 : blocks)), dim3(kBlock), 0, st, dW, elems);
    return launch_status();
}

// Up to kTableMax tensors per launch: a workgroup finds its tensor by its first-workgroup table.
struct FillTable {
    int n;
    int begin[kTableMax + 1];
    float *dst[kTableMax];
    long elems[kTableMax];
    uint64_t offset[kTableMax];
};

__device__ __forceinline__ int table_entry(const FillTable &t)
{
    int it = 0;
    for (int i = 1; i < t.n; ++i) it += (int)blockIdx.x >= t.begin[i];
    return it;
}

__global__ __launch_bounds__(kBlock) void fill_zero_table(const FillTable t)
{
    const int it = table_entry(t);
    zero_block(t.dst[it], t.elems[it], (long)((int)blockIdx.x - t.begin[it]));
}

int launch_zero_table(float *const *dW, const long *elems, int n, hipStream_t st)
{
    FillTable t{};
    t.n = n;
    long blocks = 0;
    for (int i = 0; i < n; ++i) {
        t.dst[i] = dW[i]; t.elems[i] = elems[i]; t.begin[i] = (int)blocks;
        blocks += (elems[i] + kZeroPerBlock - 1) / kZeroPerBlock;
    }
    if (blocks >= (1l << 31)) return WGRAD_UNSUPPORTED;
    t.begin[n] = (int)blocks;
    WGRAD_LAUNCH(fill_zero_table, dim3((unsigned)blocks), dim3(kBlock), 0, st, t);
    return launch_status();
}

// Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of two 32x32->64
// multiplications with the key bumped by the Weyl constants after each round.
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&o)[4])
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    o[0] = c0; o[1] = c1; o[2] = c2; o[3] = c3;
}

// The four values of generator call c: stream positions 4c .. 4c+3.  Words (0,1) and (2,3) are two
// Box-Muller pairs, u = ((word >> 8) + 0.5) / 2^24 (strictly inside (0,1)); a pair gives
// sigma * sqrt(-2 ln u1) * cos(2 pi u2) for the even position and the sine for the odd one.
__device__ __forceinline__ void normal4_at(uint64_t c, float sigma, uint64_t seed, float (&z)[4])
{
    uint32_t w[4];
    philox4x32_10((uint32_t)c, (uint32_t)(c >> 32), 0u, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), w);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        // k + 0.5 is exact in fp32 only for k < 2^23; the upper half of the range is taken from the other end,
        // u = 1 - (m + 0.5) / 2^24 with m = 2^24 - 1 - k < 2^23, which is exact again: ln u = ln(1 - (m + 0.5) / 2^24)
        // (near u = 1, where the radius is small, a rounded u would cost the radius four digits), and the
        // angle 2 pi u is the angle -2 pi (m + 0.5) / 2^24
        const uint32_t k1 = w[2 * p] >> 8, k2 = w[2 * p + 1] >> 8;
        const bool hi1 = k1 >= (1u << 23), hi2 = k2 >= (1u << 23);
        const float f1 = ((float)(hi1 ? 16777215u - k1 : k1) + 0.5f) * (1.0f / 16777216.0f);
        const float f2 = ((float)(hi2 ? 16777215u - k2 : k2) + 0.5f) * (1.0f / 16777216.0f);
        // ln(1 - f1): below 2^-7 the series (its fifth-order term is under 1e-9 of the first), above it the
        // rounding of 1 - f1 no longer matters to a radius of 0.125 and more
        const float series = -f1 * (1.0f + f1 * (0.5f + f1 * ((1.0f / 3.0f) + f1 * 0.25f)));
        const float lg = logf(hi1 ? 1.0f - f1 : f1);
        const float ln_u1 = hi1 && f1 < 0.0078125f ? series : lg;
        const float radius = sigma * sqrtf(-2.0f * ln_u1);
        float sn, cs;
        sincospif(2.0f * f2, &sn, &cs);
        z[2 * p] = radius * cs;
        z[2 * p + 1] = radius * (hi2 ? -sn : sn);
    }
}

// One thread per generator call: positions 4c..4c+3 of the stream, those of them that lie in
// [offset, offset + elems) written to dW[position - offset] (the first and the last call of a tensor may
// reach outside it).
__device__ __forceinline__ void fill_normal_call(float *__restrict__ dW, long elems, uint64_t offset, long call,
                                                 float sigma, uint64_t seed)
{
    const uint64_t c = (offset >> 2) + (uint64_t)call;
    const long first = (long)(4 * c - offset);            // index in dW of position 4c (negative for the first call of an unaligned offset)
    if (first >= elems) return;
    float z[4];
    normal4_at(c, sigma, seed, z);
    if (first >= 0 && first + 3 < elems && ((uintptr_t)(dW + first) % 16) == 0) {
        *(float4 *)(dW + first) = make_float4(z[0], z[1], z[2], z[3]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (first + j >= 0 && first + j < elems) dW[first + j] = z[j];
    }
}

// generator calls that cover positions offset .. offset + elems - 1
__host__ __device__ inline long normal_calls(long elems, uint64_t offset)
{
    return elems > 0 ? (long)(((offset + (uint64_t)elems - 1) >> 2) - (offset >> 2) + 1) : 0;
}

__global__ __launch_bounds__(kBlock) void fill_normal(float *__restrict__ dW, long elems, float sigma,
                                                      uint64_t seed, uint64_t offset)
{
    const long call = (long)blockIdx.x * kBlock + threadIdx.x;
    if (call >= normal_calls(elems, offset)) return;
    fill_normal_call(dW, elems, offset, call, sigma, seed);
}

__global__ __launch_bounds__(kBlock) void fill_normal_table(const FillTable t, float sigma, uint64_t seed)
{
    const int it = table_entry(t);
    const long call = (long)((int)blockIdx.x - t.begin[it]) * kBlock + threadIdx.x;
    if (call >= normal_calls(t.elems[it], t.offset[it])) return;
    fill_normal_call(t.dst[it], t.elems[it], t.offset[it], call, sigma, seed);
}

int launch_random_table(float *const *dW, const long *elems, const uint64_t *offset, int n, float sigma,
                        uint64_t seed, hipStream_t st)
{
    FillTable t{};
    t.n = n;
    long blocks = 0;
    for (int i = 0; i < n; ++i) {
        t.dst[i] = dW[i]; t.elems[i] = elems[i]; t.offset[i] = offset[i]; t.begin[i] = (int)blocks;
        blocks += (normal_calls(elems[i], offset[i]) + kBlock - 1) / kBlock;
    }
    if (blocks >= (1l << 31)) return WGRAD_UNSUPPORTED;
    t.begin[n] = (int)blocks;
    WGRAD_LAUNCH(fill_normal_table, dim3((unsigned)blocks), dim3(kBlock), 0, st, t, sigma, seed);
    return launch_status();
}

int launch_random(float *dW, long elems, float sigma, uint64_t seed, uint64_t offset, hipStream_t st)
{
    WGRAD_LAUNCH(fill_normal, dim3((unsigned)((normal_calls(elems, offset) + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                       dW, elems, sigma, seed, offset);
    return launch_status();
}

}  // namespace wgrad
