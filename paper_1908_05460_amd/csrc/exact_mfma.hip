// Exact filter gradient as an implicit GEMM on the CDNA4 matrix cores.
//
//   dW[k, (c,r,s)] = sum over (n,h,w) of dY[n,k,h,w] * X[n,c,h*sh + r - ph, w*sw + s - pw]
//
// (Section 2.4 of arXiv 1908.05460: the filter gradient is the input convolved with
// the output gradient.)  GEMM view: M = K output channels, columns = C*R*S filter
// taps, reduction = N*Ho*Wo output positions.  The reduction index is the
// contiguous one of both operands in NCHW, so a workgroup stages
//   - a tile of dY  [KT channels][Q positions]           and
//   - the zero-haloed input window those positions see   [channels][images][rows][cols]
// in LDS; every filter tap then reads the same staged window at a constant offset,
// and no im2col matrix ever exists.  The K x C*R*S result is far smaller than the
// reduction is long, so the reduction is split over workgroups; each keeps its
// accumulators in registers across all of its tiles and writes one partial result.
//
// MFMA: v_mfma_f32_16x16x4_f32.  Lane l supplies A[i = l%16][kk = l/16] and
// B[kk = l/16][j = l%16]; the 4 reduction slots kk are 4 consecutive staged
// positions.  The accumulator registers v = 0..3 of lane l hold D[4*(l/16) + v][l%16].
#include "common.hpp"

namespace wgrad {

typedef float float4_t __attribute__((ext_vector_type(4)));

struct ExactParams {
    const void *X, *dY;
    float *out;                 // dW when splits == 1, else partials [splits][K][C*R*S]
    Geometry g;
    int tap_mode, ktiles, ctiles, splits;
    int nti, ht, q, qpad, qp, iht, iwt, pp, ctch, h_tiles, n_groups;
    int seg;                    // ht * Wo : contiguous dY elements per (image, channel) in a tile
    int plane;                  // nti * iht * iwt : staged input elements per channel
    FastDiv d_segv, d_nsegv;    // dY staging: vectors per segment, per channel row
    FastDiv d_plane, d_img, d_iwt;  // X staging
};

template <bool BF16>
__device__ __forceinline__ float load_elem(const void *p, long i)
{
    if (BF16) return bf16_bits_to_float(((const uint16_t *)p)[i]);
    return ((const float *)p)[i];
}

template <bool BF16>
__device__ __forceinline__ float4_t load_vec4(const void *p, long i)   // i is a multiple of 4
{
    float4_t v;
    if (BF16) {
        const uint2 raw = *(const uint2 *)((const uint16_t *)p + i);
        v.x = __uint_as_float(raw.x << 16);
        v.y = __uint_as_float(raw.x & 0xffff0000u);
        v.z = __uint_as_float(raw.y << 16);
        v.w = __uint_as_float(raw.y & 0xffff0000u);
    } else {
        v = *(const float4_t *)((const float *)p + i);
    }
    return v;
}

// NT: 16-column MFMA tiles per wavefront; WK: wavefronts along K (tile of 16*WK
// output channels), the other 4/WK wavefronts split the staged positions; VEC:
// elements per dY staging access.
template <int NT, int WK, bool BF16, int VEC>
__global__ __launch_bounds__(kBlock) void wgrad_exact_mfma(const ExactParams p)
{
    constexpr int KT = 16 * WK, WQ = 4 / WK;
    extern __shared__ float smem[];
    float *dYs = smem;                              // [KT][qp]
    float *Xs = dYs + KT * p.qp;                    // [ctch][pp]
    int *xoff = (int *)(Xs + p.ctch * p.pp);        // [qpad]

    const Geometry &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wq = wave / WK;
    const int i16 = lane & 15, kk = lane >> 4;
    const int RS = g.R * g.S, CRS = g.C * RS;

    const int logical = xcd_contiguous_id(blockIdx.x, gridDim.x);
    const int coltile = logical % p.ctiles;
    const int ktile = (logical / p.ctiles) % p.ktiles;
    const int split = logical / (p.ctiles * p.ktiles);
    const int k0 = ktile * KT;

    // Column mapping. tap_mode: tile t covers 16 consecutive channels at one filter
    // tap (bank-conflict-free operand reads); otherwise 16 consecutive flat columns
    // c*R*S + r*S + s (any C, R, S).
    int coloff[NT], outcol[NT];
    int c_first;
    if (p.tap_mode) {
        c_first = coltile * 16 * (NT / RS);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int c_l = (t / RS) * 16 + i16, tap = t % RS;
            const bool ok = c_first + c_l < g.C;
            coloff[t] = ok ? c_l * p.pp + (tap / g.S) * p.iwt + tap % g.S : 0;
            outcol[t] = ok ? (c_first + c_l) * RS + tap : -1;
        }
    } else {
        const int col0 = coltile * NT * 16;
        c_first = col0 / RS;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int col = col0 + t * 16 + i16;
            const bool ok = col < CRS;
            const int c = col / RS, tap = col % RS;
            coloff[t] = ok ? (c - c_first) * p.pp + (tap / g.S) * p.iwt + tap % g.S : 0;
            outcol[t] = ok ? col : -1;
        }
    }

    // Offset of staged position q inside a staged input channel (constant for the kernel).
    for (int q = tid; q < p.qpad; q += kBlock) {
        int off = 0;
        if (q < p.q) {
            const int n_l = q / p.seg, rem = q % p.seg;
            off = n_l * p.iht * p.iwt + (rem / g.Wo) * g.sh * p.iwt + (rem % g.Wo) * g.sw;
        }
        xoff[q] = off;
    }
    // dY columns q..qpad of every row are never staged: they must read as zero.
    if (p.qpad > p.q)
        for (int e = tid; e < KT * (p.qpad - p.q); e += kBlock)
            dYs[(e / (p.qpad - p.q)) * p.qp + p.q + e % (p.qpad - p.q)] = 0.f;

    float4_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int tiles_total = p.h_tiles * p.n_groups;
    const int wt_begin = (int)((long)split * tiles_total / p.splits);
    const int wt_end = (int)((long)(split + 1) * tiles_total / p.splits);

    const int a_row = (wk * 16 + i16) * p.qp;
    const int steps = p.qpad >> 2;

    for (int wt = wt_begin; wt < wt_end; ++wt) {
        const int n0 = (wt / p.h_tiles) * p.nti, h0 = (wt % p.h_tiles) * p.ht;
        __syncthreads();   // everyone is done reading the previous tile (and xoff is written)

        // ---- stage dY[k0..k0+KT, n0..n0+nti, h0..h0+ht, :] ----
        {
            const int segv = p.seg / VEC;
            const int valid = (g.Ho - h0 < p.ht ? g.Ho - h0 : p.ht) * g.Wo;   // elements of the segment inside the map
            const int total = KT * p.nti * segv;
            for (int e = tid; e < total; e += kBlock) {
                uint32_t k_l, rem, n_l, ev;
                p.d_nsegv.divmod(e, k_l, rem);
                p.d_segv.divmod(rem, n_l, ev);
                const int k = k0 + k_l, n = n0 + n_l, el = ev * VEC;
                float *dst = dYs + k_l * p.qp + n_l * p.seg + el;
                const bool ok = k < g.K && n < g.N && el < valid;
                const long src = (((long)n * g.K + k) * g.Ho + h0) * g.Wo + el;
                if (VEC == 4) {
                    float4_t v = float4_t{0.f, 0.f, 0.f, 0.f};
                    if (ok) v = load_vec4<BF16>(p.dY, src);
                    *(float4_t *)dst = v;
                } else {
                    *dst = ok ? load_elem<BF16>(p.dY, src) : 0.f;
                }
            }
        }
        // ---- stage the input window, zero outside X (padding, ragged edges) ----
        {
            const int total = p.ctch * p.plane;
            const int ih0 = h0 * g.sh - g.ph;
            for (int e = tid; e < total; e += kBlock) {
                uint32_t c_l, rem, n_l, rem2, ih_l, iw_l;
                p.d_plane.divmod(e, c_l, rem);
                p.d_img.divmod(rem, n_l, rem2);
                p.d_iwt.divmod(rem2, ih_l, iw_l);
                const int c = c_first + c_l, n = n0 + n_l, ih = ih0 + (int)ih_l, iw = (int)iw_l - g.pw;
                float v = 0.f;
                if (c < g.C && n < g.N && ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)
                    v = load_elem<BF16>(p.X, (((long)n * g.C + c) * g.H + ih) * g.W + iw);
                Xs[c_l * p.pp + rem] = v;
            }
        }
        __syncthreads();

        // ---- contract: 4 positions per MFMA step, NT column tiles per A operand ----
#pragma unroll 2
        for (int t = wq; t < steps; t += WQ) {
            const int q = 4 * t + kk;
            const float a = dYs[a_row + q];
            const int xo = xoff[q];
            float b[NT];
#pragma unroll
            for (int j = 0; j < NT; ++j) b[j] = Xs[coloff[j] + xo];
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[j], acc[j], 0, 0, 0);
        }
    }

    // ---- wavefronts that split the positions add their accumulators through LDS ----
    if (WQ > 1) {
        __syncthreads();
        float4_t *red = (float4_t *)smem;   // [(WQ-1)][WK][NT][64]
        if (wq > 0) {
#pragma unroll
            for (int j = 0; j < NT; ++j) red[(((wq - 1) * WK + wk) * NT + j) * 64 + lane] = acc[j];
        }
        __syncthreads();
        if (wq == 0) {
            for (int w = 0; w < WQ - 1; ++w)
#pragma unroll
                for (int j = 0; j < NT; ++j) acc[j] += red[((w * WK + wk) * NT + j) * 64 + lane];
        }
    }
    if (wq == 0) {
        float *out = p.out + (long)split * g.K * CRS;
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            if (outcol[j] < 0) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int k = k0 + wk * 16 + 4 * kk + v;
                if (k < g.K) out[(long)k * CRS + outcol[j]] = acc[j][v];
            }
        }
    }
}

// ------------------------------------------------------------------------------------
// Host side: tile plan and launch.
// ------------------------------------------------------------------------------------
#ifndef WGRAD_EXACT_KQ       // target number of staged dY elements (KT * Q) per tile
#define WGRAD_EXACT_KQ 8192
#endif
#ifndef WGRAD_EXACT_BLOCKS   // workgroups to aim for when splitting the reduction
#define WGRAD_EXACT_BLOCKS 1024
#endif
constexpr size_t kMaxLds = 64 * 1024;

static int pitch_mod32(int len, int want, int multiple)
{
    // smallest pitch >= len with pitch % 32 == want (want is a multiple of `multiple`)
    int p = (len + multiple - 1) / multiple * multiple;
    while (p % 32 != want) p += multiple;
    return p;
}

ExactPlan plan_exact(const Geometry &g)
{
    ExactPlan pl{};
    const int RS = g.R * g.S;
    const long CRS = g.crs();
    pl.wk = g.K <= 16 ? 1 : (g.K <= 32 ? 2 : 4);
    const int KT = 16 * pl.wk;
    if (g.C % 16 == 0 && RS == 9) { pl.tap_mode = 1; pl.nt = 9; }
    else if (g.C % 64 == 0 && RS == 1) { pl.tap_mode = 1; pl.nt = 4; }
    else {
        pl.tap_mode = 0;
        pl.nt = CRS <= 32 ? 2 : (CRS <= 64 ? 4 : 9);
    }
    pl.ktiles = (g.K + KT - 1) / KT;
    if (pl.tap_mode) {
        const int ct = 16 * (pl.nt / RS);
        pl.ctiles = (g.C + ct - 1) / ct;
        pl.ctch = ct;
    } else {
        const int cols = pl.nt * 16;
        pl.ctiles = (int)((CRS + cols - 1) / cols);
        pl.ctch = (cols - 1) / RS + 2;
        if (pl.ctch > g.C) pl.ctch = g.C;
    }

    const int L = g.Ho * g.Wo;
    for (int qt = WGRAD_EXACT_KQ / KT; qt >= 4; qt /= 2) {
        if (L >= qt) { pl.nti = 1; pl.ht = qt / g.Wo < 1 ? 1 : qt / g.Wo; if (pl.ht > g.Ho) pl.ht = g.Ho; }
        else { pl.ht = g.Ho; pl.nti = qt / L < 1 ? 1 : qt / L; if (pl.nti > g.N) pl.nti = g.N; }
        pl.q = pl.nti * pl.ht * g.Wo;
        pl.qpad = (pl.q + 3) / 4 * 4;
        pl.qp = pitch_mod32(pl.qpad, 4, 4);
        pl.iht = (pl.ht - 1) * g.sh + g.R;
        pl.iwt = (g.Wo - 1) * g.sw + g.S;
        pl.pp = pitch_mod32(pl.nti * pl.iht * pl.iwt, 2, 1);
        size_t lds = ((size_t)KT * pl.qp + (size_t)pl.ctch * pl.pp + pl.qpad) * 4;
        const size_t red = (size_t)(4 / pl.wk - 1) * pl.wk * pl.nt * 64 * 16;
        if (red > lds) lds = red;
        pl.lds_bytes = lds;
        if (lds <= kMaxLds) { pl.ok = true; break; }
    }
    if (!pl.ok) return pl;
    // fast-division bounds: dividend * divisor < 2^32
    const long plane = (long)pl.nti * pl.iht * pl.iwt;
    if ((long)pl.ctch * plane * plane >= (1ll << 32) || (long)KT * pl.q * pl.q >= (1ll << 32)) { pl.ok = false; return pl; }

    pl.h_tiles = (g.Ho + pl.ht - 1) / pl.ht;
    pl.n_groups = (g.N + pl.nti - 1) / pl.nti;
    const long tiles = (long)pl.h_tiles * pl.n_groups;
    long out_tiles = (long)pl.ktiles * pl.ctiles;
    long splits = (WGRAD_EXACT_BLOCKS + out_tiles - 1) / out_tiles;
    if (splits > tiles) splits = tiles;
    if (splits < 1) splits = 1;
    pl.splits = (int)splits;

    const int seg = pl.ht * g.Wo;
    const bool tail = g.Ho % pl.ht != 0;
    pl.vec = (seg % 4 == 0 && L % 4 == 0 && (!tail || g.Wo % 4 == 0)) ? 4 : 1;
    pl.ws_bytes = pl.splits > 1 ? align_up((size_t)pl.splits * g.dw_elems() * 4) : 0;
    return pl;
}

template <int NT, int WK, bool BF16, int VEC>
static void launch_inst(const ExactParams &p, int grid, size_t lds, hipStream_t st)
{
    WGRAD_LAUNCH((wgrad_exact_mfma<NT, WK, BF16, VEC>), dim3(grid), dim3(kBlock), lds, st, p);
}

template <int NT, int WK>
static void launch_dtype(const ExactParams &p, int grid, size_t lds, int vec, hipStream_t st)
{
    if (p.g.bf16) { if (vec == 4) launch_inst<NT, WK, true, 4>(p, grid, lds, st); else launch_inst<NT, WK, true, 1>(p, grid, lds, st); }
    else          { if (vec == 4) launch_inst<NT, WK, false, 4>(p, grid, lds, st); else launch_inst<NT, WK, false, 1>(p, grid, lds, st); }
}

template <int NT>
static void launch_wk(const ExactParams &p, int wk, int grid, size_t lds, int vec, hipStream_t st)
{
    if (wk == 1) launch_dtype<NT, 1>(p, grid, lds, vec, st);
    else if (wk == 2) launch_dtype<NT, 2>(p, grid, lds, vec, st);
    else launch_dtype<NT, 4>(p, grid, lds, vec, st);
}

int launch_exact(const Geometry &g, const ExactPlan &pl, const void *X, const void *dY, float *dW,
                 void *ws, hipStream_t st)
{
    ExactParams p{};
    p.X = X; p.dY = dY;
    p.out = pl.splits > 1 ? (float *)ws : dW;
    p.g = g;
    p.tap_mode = pl.tap_mode; p.ktiles = pl.ktiles; p.ctiles = pl.ctiles; p.splits = pl.splits;
    p.nti = pl.nti; p.ht = pl.ht; p.q = pl.q; p.qpad = pl.qpad; p.qp = pl.qp;
    p.iht = pl.iht; p.iwt = pl.iwt; p.pp = pl.pp; p.ctch = pl.ctch;
    p.h_tiles = pl.h_tiles; p.n_groups = pl.n_groups;
    p.seg = pl.ht * g.Wo;
    p.plane = pl.nti * pl.iht * pl.iwt;
    // the 16-byte dY staging path also needs 16-byte aligned tensors
    int vec = pl.vec;
    if (vec == 4 && ((uintptr_t)dY % (g.bf16 ? 8 : 16)) != 0) vec = 1;
    p.d_segv = FastDiv(p.seg / vec);
    p.d_nsegv = FastDiv(pl.nti * (p.seg / vec));
    p.d_plane = FastDiv(p.plane);
    p.d_img = FastDiv(pl.iht * pl.iwt);
    p.d_iwt = FastDiv(pl.iwt);

    const int grid = pl.ktiles * pl.ctiles * pl.splits;
    switch (pl.nt) {
        case 2: launch_wk<2>(p, pl.wk, grid, pl.lds_bytes, vec, st); break;
        case 4: launch_wk<4>(p, pl.wk, grid, pl.lds_bytes, vec, st); break;
        default: launch_wk<9>(p, pl.wk, grid, pl.lds_bytes, vec, st); break;
    }
    int rc = launch_status();
    if (rc != WGRAD_OK) return rc;
    if (pl.splits > 1) return launch_combine((const float *)ws, pl.splits, g.dw_elems(), 1.0f, dW, st);
    return WGRAD_OK;
}

}  // namespace wgrad
