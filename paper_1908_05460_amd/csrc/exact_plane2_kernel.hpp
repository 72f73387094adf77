// Exact filter gradient of 3x3, stride-1, padding-1 layers on 2x2 planes (fp32), as ONE plain matrix product.
//
// On a 2x2 plane every output position sees every input element of its plane through exactly one tap, and
// five of the nine taps of a position fall into the padding.  The definition (Section 2.4)
//     dW[k,c,r,s] = sum_{n,h,w} dY[n,k,h,w] * X[n,c,h+r-1,w+s-1]
// therefore regroups, with p = (h,w) and e = (ih,iw) running over the four positions / elements of a plane, into
//     G[(k,p),(c,e)] = sum_n dY[n,k,p] * X[n,c,e]                 -- a [4K x N] x [N x 4C] product
//     dW[k,c,r,s]    = sum of G[(k,p),(c,e)] over the (p,e) with ih-h+1 = r, iw-w+1 = s   (16 terms -> 9 taps)
// which multiplies no padding at all: 16 multiply-adds per (n,k,c) instead of the 36 of the implicit GEMM over
// taps.  dY viewed as [N][4K] and X as [N][4C] are both contiguous with the reduction index n slowest.
//
// Matrix instruction v_mfma_f32_16x16x4_f32 (lane l supplies A[l%16][l/16], B[l/16][l%16]; holds D[4(l/16)+t][l%16]):
//   - lane (i, kk) loads the 16 bytes dY[4s+kk][k0+i][0..3]: element v is the A operand of "row tile v", whose
//     row i is (channel k0+i, position v); likewise X[4s+kk][c0+j][0..3] gives the B operands of four column
//     tiles.  One 16-byte load per operand feeds 16 matrix instructions (a 64x64 tile of G per wavefront), and
//     nothing passes through LDS.
//   - afterwards a lane holds, for its four channels k0+4(l/16)+t and its channel c0+l%16, all sixteen (p,e)
//     terms: the fold to nine taps is local to the lane, and it writes 36 contiguous bytes per (k,c).
// The reduction is only N deep, so no split and no partial sums: a wavefront per 16x16 block of (k,c).
#pragma once
#include "exact_stream_kernel.hpp"

namespace wgrad {

constexpr int kPlane2Prefetch = 4;   // reduction steps (four images each) whose operands are in flight

// p: the tensors, the geometry and per_prob (workgroups per problem) of the launch parameters are used;
// bid: the workgroup's number among the per_prob * problems of its launch (or of its group in a multi-shape launch).
__device__ __forceinline__ void plane2_body(const StreamShape &p, const void *const *Xt, const void *const *dYt, float *const *outt, int bid)
{
    const int lane = threadIdx.x & 63;
    const int prob = bid / p.per_prob;
    const int ctiles = p.g.C / 16, tiles = (p.g.K / 16) * ctiles;
    const int tile = (bid - prob * p.per_prob) * (kBlock / 64) + (int)__builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (tile >= tiles) return;                                   // wavefront-uniform; the body has no barrier
    const int k0 = (tile / ctiles) * 16, c0 = (tile % ctiles) * 16;
    const int i16 = lane & 15, kk = lane >> 4;
    const char *__restrict__ dYb = (const char *)dYt[prob];
    const char *__restrict__ Xb = (const char *)Xt[prob];
    const int N = p.g.N;

    // byte offsets of this lane's pieces in reduction step s: image n = 4s + kk (clamped; its values are then zeroed)
    const uint32_t a_lane = (uint32_t)(k0 + i16) * 16u, b_lane = (uint32_t)(c0 + i16) * 16u;
    const uint32_t a_img = (uint32_t)p.g.K * 16u, b_img = (uint32_t)p.g.C * 16u;
    const int steps = (N + 3) / 4;
    auto load = [&](int s, float4_t &a, float4_t &b) {
        const int n = 4 * s + kk;
        const bool live = n < N;
        const uint32_t nc = (uint32_t)(live ? n : N - 1);
        a = *(const float4_t *)(dYb + nc * a_img + a_lane);
        b = *(const float4_t *)(Xb + nc * b_img + b_lane);
        if (!live) { a = float4_t{0.f, 0.f, 0.f, 0.f}; b = a; }
    };

    float4_t acc[4][4];
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[v][u] = float4_t{0.f, 0.f, 0.f, 0.f};

    constexpr int PF = kPlane2Prefetch;
    float4_t ra[PF], rb[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q) load(q, ra[q], rb[q]);
    for (int s0 = 0; s0 < steps; s0 += PF) {
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            const float4_t a = ra[q], b = rb[q];
            load(s0 + q + PF, ra[q], rb[q]);                     // a step beyond the batch loads zeros
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    acc[v][u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[v], b[u], acc[v][u], 0, 0, 0);
        }
    }

    // fold: position p = 2h + w, element e = 2ih + iw contribute to tap (ih - h + 1, iw - w + 1)
    float *__restrict__ out = outt[prob];
    const int c = c0 + i16;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int k = k0 + 4 * kk + t;
        float tap[9];
#pragma unroll
        for (int x = 0; x < 9; ++x) tap[x] = 0.f;
#pragma unroll
        for (int pp = 0; pp < 4; ++pp)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int r = (e >> 1) - (pp >> 1) + 1, s = (e & 1) - (pp & 1) + 1;
                tap[r * 3 + s] += acc[pp][e][t];
            }
        float *o = out + ((long)k * p.g.C + c) * 9;
#pragma unroll
        for (int x = 0; x < 9; ++x) o[x] = tap[x];
    }
}

}  // namespace wgrad
