// General form of the exact filter gradient (arXiv 1908.05460, Section 2.1: the gradient the
// approximation replaces): dW[k,c,r,s] = sum over images and output positions of
// dY[n,k,ho,wo] * X[n,c,ho*sh+r-ph,wo*sw+s-pw], taps outside X contributing nothing.
//
// This is the form for the shapes that the tiled matrix-core kernels do not take (their tiles
// hold whole output rows, so very wide or widely strided inputs do not fit the LDS).  It makes
// no assumption about the shape or about alignment: a 64 x 64 tile of dW per workgroup, the
// reduction over the N*Ho*Wo positions cut into 16-position steps whose dY values and input
// taps are gathered element by element into LDS, fp32 multiply-adds on the vector unit, the
// reduction range split over workgroups whose partial results the common reduction adds.
#include "common.hpp"

namespace wgrad {

namespace {

constexpr int kDT = 64;              // tile edge of dW (output channels x entries per channel)
constexpr int kDP = 16;              // positions per step
constexpr int kDPitch = kDT + 4;     // LDS row pitch in floats

struct DirectParams {
    const void *X;
    const void *dY;
    float *out;                      // [splits][K][C*R*S]
    Geometry g;
    int ktiles, jtiles;
    long steps, steps_per_split;     // 16-position steps in all and per workgroup
};

template <bool BF16>
__device__ __forceinline__ float load_elem(const void *p, long i)
{
    return BF16 ? bf16_bits_to_float(((const uint16_t *)p)[i]) : ((const float *)p)[i];
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void wgrad_exact_direct(DirectParams p)
{
    __shared__ __align__(16) float As[kDP][kDPitch];   // dY:   [position][output channel]
    __shared__ __align__(16) float Bs[kDP][kDPitch];   // taps: [position][entry]
    const Geometry &g = p.g;
    const int tid = threadIdx.x;
    const int tile = blockIdx.x, split = blockIdx.y;
    const int k0 = (tile % p.ktiles) * kDT, j0 = (tile / p.ktiles) * kDT;
    const int L = g.Ho * g.Wo, RS = g.R * g.S, CRS = g.C * RS;
    const long P = (long)g.N * L;

    // staging role: position pcol of the step, rows row + 16*i of both tiles
    const int pcol = tid & 15, row = tid >> 4;
    int tc[4], tr[4], ts[4];                      // channel and tap of the entries this thread gathers
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = j0 + row + 16 * i;
        tc[i] = j < CRS ? j / RS : -1;
        tr[i] = (j % RS) / g.S;
        ts[i] = j % g.S;
    }
    // compute role: a 4 x 4 block of the tile
    const int ty = tid >> 4, tx = tid & 15;
    float acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = 0.f;

    const long s_begin = (long)split * p.steps_per_split;
    long s_end = s_begin + p.steps_per_split;
    if (s_end > p.steps) s_end = p.steps;
    for (long step = s_begin; step < s_end; ++step) {
        const long pos = step * kDP + pcol;
        float a_val[4], b_val[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a_val[i] = b_val[i] = 0.f;
        if (pos < P) {
            const long n = pos / L;
            const int l = (int)(pos - n * L);
            const int ho = l / g.Wo, wo = l - ho * g.Wo;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = k0 + row + 16 * i;
                if (k < g.K) a_val[i] = load_elem<BF16>(p.dY, (n * g.K + k) * L + l);
                const int ih = ho * g.sh + tr[i] - g.ph, iw = wo * g.sw + ts[i] - g.pw;
                if (tc[i] >= 0 && ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)
                    b_val[i] = load_elem<BF16>(p.X, ((n * g.C + tc[i]) * g.H + ih) * g.W + iw);
            }
        }
        __syncthreads();                          // the previous step's tiles have been consumed
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            As[pcol][row + 16 * i] = a_val[i];
            Bs[pcol][row + 16 * i] = b_val[i];
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kDP; ++q) {
            const float4 a4 = *(const float4 *)&As[q][4 * ty];
            const float4 b4 = *(const float4 *)&Bs[q][4 * tx];
            const float av[4] = {a4.x, a4.y, a4.z, a4.w}, bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[a][b] = fmaf(av[a], bv[b], acc[a][b]);
        }
    }
    float *out = p.out + (long)split * g.K * CRS;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const int k = k0 + 4 * ty + a;
        if (k >= g.K) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int j = j0 + 4 * tx + b;
            if (j < CRS) out[(long)k * CRS + j] = acc[a][b];
        }
    }
}

}  // namespace

// Fills the plan fields the general form uses: its output tiles and the number of workgroups
// the reduction over the positions is split into.
void plan_exact_direct(const Geometry &g, ExactPlan &pl)
{
    pl.direct = 1;
    pl.stream = pl.mm16 = 0;
    pl.ktiles = (g.K + kDT - 1) / kDT;
    pl.ctiles = (int)((g.crs() + kDT - 1) / kDT);
    const long steps = ((long)g.N * g.Ho * g.Wo + kDP - 1) / kDP;
    const long tiles = (long)pl.ktiles * pl.ctiles;
    long splits = (4 * kNumCU + tiles - 1) / tiles;            // four workgroups per CU
    if (splits > steps / 8) splits = steps / 8;                 // at least eight steps each
    if (splits > 1024) splits = 1024;
    if (splits < 1) splits = 1;
    pl.splits = (int)splits;
    pl.lds_bytes = 2 * kDP * kDPitch * sizeof(float);
    pl.ws_bytes = pl.splits > 1 ? align_up((size_t)pl.splits * g.dw_elems() * sizeof(float)) : 0;
    pl.ok = tiles < (1l << 31);
}

int launch_exact_direct(const Geometry &g, const ExactPlan &pl, const void *X, const void *dY, float *dW, void *ws,
                        hipStream_t st, CombineQueue *defer)
{
    DirectParams p{};
    p.X = X; p.dY = dY;
    p.out = pl.splits > 1 ? (float *)ws : dW;
    p.g = g;
    p.ktiles = pl.ktiles; p.jtiles = pl.ctiles;
    p.steps = ((long)g.N * g.Ho * g.Wo + kDP - 1) / kDP;
    p.steps_per_split = (p.steps + pl.splits - 1) / pl.splits;
    const dim3 grid((unsigned)(pl.ktiles * pl.ctiles), (unsigned)pl.splits);
    if (g.bf16) WGRAD_LAUNCH((wgrad_exact_direct<true>), grid, dim3(kBlock), 0, st, p);
    else        WGRAD_LAUNCH((wgrad_exact_direct<false>), grid, dim3(kBlock), 0, st, p);
    const int rc = launch_status();
    if (rc != WGRAD_OK || pl.splits == 1) return rc;
    float *dst[1] = {dW};
    return launch_combine((const float *)ws, 0, pl.splits, g.dw_elems(), 1.0f, dst, 1, st, defer);
}

}  // namespace wgrad
