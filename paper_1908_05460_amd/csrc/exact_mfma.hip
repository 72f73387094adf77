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
// Pipeline (vector staging modes): while the wavefronts contract tile t out of LDS,
// the 16-byte global loads of tile t+1 are already in flight into registers; they are
// written to LDS after the barrier that ends tile t.  Which element of a tile a thread
// stages is the same for every tile, so each thread decodes its staging slots once
// (LDS destination, offset from the tile origin) and keeps them in registers.  The
// contraction loop itself is unrolled by two with the LDS operand reads of step i+1
// issued before the MFMAs of step i.
//
// MFMA: v_mfma_f32_16x16x4_f32.  Lane l supplies A[i = l%16][kk = l/16] and
// B[kk = l/16][j = l%16]; the 4 reduction slots kk are 4 consecutive staged
// positions.  The accumulator registers v = 0..3 of lane l hold D[4*(l/16) + v][l%16].
#include "exact_common.hpp"

namespace wgrad {

// Staging slots per thread and tile (16-byte loads of dY; 16- or 8-byte loads of X).  Narrow K
// tiles have few dY rows but the same input window, so they trade dY slots for X slots.
__host__ __device__ constexpr int slots_dy(int wk) { return wk == 1 ? 4 : 8; }
__host__ __device__ constexpr int slots_x(int wk) { return wk == 4 ? 4 : 6; }

struct ExactParams {
    const void *X, *dY;
    float *out;                 // dW when splits == 1, else partials [splits][K][C*R*S]
    Geometry g;
    int tap_mode, ktiles, ctiles, splits;
    int nti, ht, q, qpad, qp, iht, iwt, pp, ctch, h_tiles, n_groups;
    int seg;                    // ht * Wo : contiguous dY elements per (image, channel) in a tile
    int plane;                  // nti * iht * iwt : staged input elements per channel
    FastDiv d_segv, d_nsegv;    // dY staging: vectors per segment, per channel row
    FastDiv d_plane, d_img, d_iwt;   // X staging, element-wise mode
    FastDiv d_wv, d_rows, d_iht;     // X staging, vector modes: vectors per row, rows per channel, rows per image
    FastDiv d_rs, d_s, d_seg, d_wo, d_htiles;
    // tap mode, per MFMA column tile: first channel (relative to the block's), LDS offset of the tap, tap index
    int tile_c0[9], tile_toff[9], tile_tap[9];
};

// Column mapping of MFMA column tile t for lane column i16.  tap_mode: the tile covers 16
// consecutive channels at one filter tap (bank-conflict-free operand reads; the per-tile
// constants come precomputed from the host); otherwise 16 consecutive flat columns
// c*R*S + r*S + s (any C, R, S).  Returns the LDS offset of the column inside the staged
// window (0 for a padding column) and the column's index local to the workgroup, in
// output order (-1 for a padding column).
template <int NT>
__device__ __forceinline__ void column_of(const ExactParams &p, int coltile, int t, int i16, int c_first,
                                          int &lds_off, int &local_col)
{
    const Geometry &g = p.g;
    const int RS = g.R * g.S;
    if (p.tap_mode) {
        const int c_l = p.tile_c0[t] + i16;
        const bool ok = c_first + c_l < g.C;
        lds_off = ok ? c_l * p.pp + p.tile_toff[t] : 0;
        local_col = ok ? c_l * RS + p.tile_tap[t] : -1;
    } else {
        const int col = coltile * NT * 16 + t * 16 + i16;
        const bool ok = col < g.C * RS;
        uint32_t c, tap, r, s;
        p.d_rs.divmod(col, c, tap);
        p.d_s.divmod(tap, r, s);
        lds_off = ok ? (int)((c - c_first) * p.pp + r * p.iwt + s) : 0;
        local_col = ok ? t * 16 + i16 : -1;
    }
}

// One tile's staging registers (vector modes).
template <bool BF16, int XV, int DS, int XS>
struct Stage {
    Vec<BF16, 4> dy[DS];
    Vec<BF16, XV> x[XS];
    uint32_t row_ok;            // bit u: the input row of X slot u lies inside X for this tile
};

// NT: 16-column MFMA tiles per wavefront; WK: wavefronts along K (tile of 16*WK output
// channels), the other 4/WK wavefronts split the staged positions.  XV: elements per
// global access when staging (4 or 2: rows of X and segments of dY are read in 16- or
// 8-byte pieces, pipelined through registers; 0: element-wise staging for shapes and
// alignments that allow nothing wider).
template <int NT, int WK, bool BF16, int XV>
__global__ __launch_bounds__(kBlock) void wgrad_exact_mfma(const ExactParams p)
{
    constexpr int KT = 16 * WK, WQ = 4 / WK;
    constexpr bool FAST = XV != 0;
    constexpr int XVn = FAST ? XV : 2;                  // placeholder width for the unused registers
    constexpr int ESZ = BF16 ? 2 : 4;                   // bytes per input element
    constexpr int NCB = NT * 16;                        // columns of the workgroup's output tile
    constexpr int kSlotsDY = slots_dy(WK), kSlotsX = slots_x(WK);
    typedef Stage<BF16, XVn, kSlotsDY, kSlotsX> StageT;
    extern __shared__ float smem[];
    float *dYs = smem;                              // [KT][qp]
    float *Xs = dYs + KT * p.qp;                    // [ctch][pp]
    int *xoff = (int *)(Xs + p.ctch * p.pp);        // [qpad + 16]

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
    const int c_first = p.tap_mode ? coltile * 16 * (NT / RS) : (coltile * NT * 16) / RS;

    TRACE(0);
    int coloff[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int lc;
        column_of<NT>(p, coltile, t, i16, c_first, coloff[t], lc);
    }

    TRACE(11);
    // Offset of staged position q inside a staged input channel (constant for the kernel);
    // 16 spare entries let the contraction loop read up to three steps ahead.
    for (int q = tid; q < p.qpad + 16; q += kBlock) {
        int off = 0;
        if (q < p.q) {
            uint32_t n_l, rem, h_l, w;
            p.d_seg.divmod(q, n_l, rem);
            p.d_wo.divmod(rem, h_l, w);
            off = n_l * p.iht * p.iwt + h_l * g.sh * p.iwt + w * g.sw;
        }
        xoff[q] = off;
    }
    TRACE(12);
    if (FAST) {
        // vector staging writes only cells that hold data: padding columns of the window,
        // channels beyond C, rows of dY beyond K and positions q..qpad are zeroed once here
        const int zn = KT * p.qp + p.ctch * p.pp;
        for (int e = tid; e < (zn >> 2); e += kBlock) ((float4_t *)smem)[e] = float4_t{0.f, 0.f, 0.f, 0.f};
        if (tid < (zn & 3)) smem[(zn & ~3) + tid] = 0.f;
    } else if (p.qpad > p.q) {
        // dY columns q..qpad of every row are never staged: they must read as zero
        for (int e = tid; e < KT * (p.qpad - p.q); e += kBlock)
            dYs[(e / (p.qpad - p.q)) * p.qp + p.q + e % (p.qpad - p.q)] = 0.f;
    }

    TRACE(13);
    float4_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int tiles_total = p.h_tiles * p.n_groups;
    const int wt_begin = (int)((long)split * tiles_total / p.splits);
    const int wt_end = (int)((long)(split + 1) * tiles_total / p.splits);

    // contraction: every wavefront owns spw consecutive steps of 4 positions; the operands of
    // the next step are read from LDS before the MFMAs of the current one are issued
    const int spw = (p.qpad >> 2) / WQ;                // even (qpad is a multiple of 8 * WQ)
    const float *a_ptr = dYs + (wk * 16 + i16) * p.qp + 4 * wq * spw + kk;
    const int *xo_ptr = xoff + 4 * wq * spw + kk;
    auto contract = [&]() {
        float a0, a1, b0[NT], b1[NT];
        int xoA = xo_ptr[0], xoB = xo_ptr[4];
        a0 = a_ptr[0];
#pragma unroll
        for (int j = 0; j < NT; ++j) b0[j] = Xs[coloff[j] + xoA];
        xoA = xo_ptr[8];
        for (int i = 0; i < spw; i += 2) {
            // the scheduling barriers keep the order written here: LDS reads of the next step are
            // issued, then the MFMAs of the current step run while those reads are in flight
            a1 = a_ptr[4 * (i + 1)];
#pragma unroll
            for (int j = 0; j < NT; ++j) b1[j] = Xs[coloff[j] + xoB];
            xoB = xo_ptr[4 * (i + 3)];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, b0[j], acc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            a0 = a_ptr[4 * (i + 2)];                 // one step past the end on the last trip: read, not used
#pragma unroll
            for (int j = 0; j < NT; ++j) b0[j] = Xs[coloff[j] + xoA];
            xoA = xo_ptr[4 * (i + 4)];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NT; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1[j], acc[j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (FAST) {
        // ---- this thread's staging slots, decoded once.  No tile is ragged in these modes (ht
        //      divides Ho, nti divides N), so a slot is either always inside the tensors or
        //      never; only the input row can fall on padding, tile by tile.  Every slot always
        //      loads (unused ones re-read the tile's first element, padding rows a clamped row),
        //      so the number of loads in flight is fixed and a tile can be waited for while the
        //      next one is still arriving. ----
        int dy_dst[kSlotsDY];        // LDS float index, -1 = slot unused
        uint32_t dy_src[kSlotsDY];   // byte offset from the tile's first dY element
        int x_pack[kSlotsX];         // LDS float index | ih_l << 20 | valid elements << 28, -1 = unused
        uint32_t x_src[kSlotsX];     // byte offset from row 0 of the tile's first (image, channel)
        {
            const int L = g.Ho * g.Wo;
            const int dy_total = KT * p.nti * (p.seg >> 2);
#pragma unroll
            for (int u = 0; u < kSlotsDY; ++u) {
                const int e = tid + u * kBlock;
                dy_dst[u] = -1; dy_src[u] = 0;
                if (e < dy_total) {
                    uint32_t k_l, rem, n_l, ev;
                    p.d_nsegv.divmod(e, k_l, rem);
                    p.d_segv.divmod(rem, n_l, ev);
                    if (k0 + (int)k_l < g.K) {
                        dy_dst[u] = k_l * p.qp + n_l * p.seg + ev * 4;
                        dy_src[u] = ((n_l * g.K + k_l) * L + ev * 4) * ESZ;
                    }
                }
            }
            const int x_total = p.ctch * p.nti * p.iht * (int)p.d_wv.d;
#pragma unroll
            for (int u = 0; u < kSlotsX; ++u) {
                const int e = tid + u * kBlock;
                x_pack[u] = -1; x_src[u] = 0;
                if (e < x_total) {
                    uint32_t row, jv, c_l, rem, n_l, ih_l;
                    p.d_wv.divmod(e, row, jv);
                    p.d_rows.divmod(row, c_l, rem);
                    p.d_iht.divmod(rem, n_l, ih_l);
                    const int col0 = g.pw + jv * XVn;            // window column of the first element
                    int nv = p.iwt - col0;                       // columns right of the window are not staged
                    nv = nv > XVn ? XVn : nv;
                    if (c_first + (int)c_l < g.C && nv > 0) {
                        x_pack[u] = (int)(c_l * p.pp + rem * p.iwt + col0) | (int)(ih_l << 20) | (nv << 28);
                        x_src[u] = ((n_l * g.C + c_l) * (g.H * g.W) + jv * XVn) * ESZ;
                    }
                }
            }
        }
        // issue the global loads of tile wt into a register stage
        auto prefetch = [&](int wt, StageT &st) {
            uint32_t ng, hti;
            p.d_htiles.divmod(wt, ng, hti);
            const int n0 = ng * p.nti, h0 = hti * p.ht;
            // uniform tile origins: the loads below are scalar base + 32-bit lane offset
            const char *dy_base = (const char *)p.dY + (((long)n0 * g.K + k0) * g.Ho + h0) * g.Wo * ESZ;
#pragma unroll
            for (int u = 0; u < kSlotsDY; ++u) st.dy[u].load(dy_base, dy_src[u]);
            const int ih0 = h0 * g.sh - g.ph;
            const char *x_base = (const char *)p.X + ((long)n0 * g.C + c_first) * g.H * g.W * ESZ;
            st.row_ok = 0;
#pragma unroll
            for (int u = 0; u < kSlotsX; ++u) {
                int ih = ih0 + ((x_pack[u] >> 20) & 0xff);
                if (ih >= 0 && ih < g.H) st.row_ok |= 1u << u;
                ih = ih < 0 ? 0 : (ih >= g.H ? g.H - 1 : ih);
                st.x[u].load(x_base, x_src[u] + ih * (g.W * ESZ));
            }
        };
        // register stage -> LDS
        auto commit = [&](const StageT &st) {
#pragma unroll
            for (int u = 0; u < kSlotsDY; ++u)
                if (dy_dst[u] >= 0) {
                    float4_t v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = st.dy[u].get(i);
                    *(float4_t *)(dYs + dy_dst[u]) = v;
                }
#pragma unroll
            for (int u = 0; u < kSlotsX; ++u)
                if (x_pack[u] >= 0) {
                    float *dst = Xs + (x_pack[u] & 0xfffff);
                    const int nv = x_pack[u] >> 28;
                    const bool ok = (st.row_ok >> u) & 1;
#pragma unroll
                    for (int i = 0; i < XVn; ++i)
                        if (i < nv) dst[i] = ok ? st.x[u].get(i) : 0.f;
                }
        };

        // two register stages: tiles wt and wt+1 are in flight while tile wt-1 is contracted
        StageT sa, sb;
        TRACE(1);
        if (wt_begin < wt_end) prefetch(wt_begin, sa);
        if (wt_begin + 1 < wt_end) prefetch(wt_begin + 1, sb);
        TRACE(2);
        for (int wt = wt_begin; wt < wt_end; wt += 2) {
            __syncthreads();   // everyone is done reading the previous tile (and the tables are written)
            if (wt == wt_begin) TRACE(3);
            commit(sa);
            __syncthreads();
            if (wt == wt_begin) TRACE(4);
            if (wt + 2 < wt_end) prefetch(wt + 2, sa);
            contract();
            if (wt == wt_begin) TRACE(5);
            if (wt + 1 < wt_end) {
                __syncthreads();
                commit(sb);
                __syncthreads();
                if (wt == wt_begin) TRACE(6);
                if (wt + 3 < wt_end) prefetch(wt + 3, sb);
                contract();
                if (wt == wt_begin) TRACE(7);
            }
        }
        TRACE(8);
    } else {
        for (int wt = wt_begin; wt < wt_end; ++wt) {
            const int n0 = (wt / p.h_tiles) * p.nti, h0 = (wt % p.h_tiles) * p.ht;
            __syncthreads();   // everyone is done reading the previous tile (and the tables are written)
            // ---- element-wise staging of dY[k0..k0+KT, n0..n0+nti, h0..h0+ht, :] ----
            {
                const int valid = (g.Ho - h0 < p.ht ? g.Ho - h0 : p.ht) * g.Wo;
                const int total = KT * p.nti * p.seg;
                for (int e0 = tid; e0 < total; e0 += 4 * kBlock) {
                    float v[4];
                    int dst[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int e = e0 + u * kBlock;
                        v[u] = 0.f; dst[u] = -1;
                        if (e < total) {
                            uint32_t k_l, rem, n_l, el;
                            p.d_nsegv.divmod(e, k_l, rem);
                            p.d_segv.divmod(rem, n_l, el);
                            const int k = k0 + k_l, n = n0 + n_l;
                            dst[u] = k_l * p.qp + n_l * p.seg + el;
                            if (k < g.K && n < g.N && (int)el < valid)
                                v[u] = load_elem<BF16>(p.dY, (((long)n * g.K + k) * g.Ho + h0) * g.Wo + el);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (dst[u] >= 0) dYs[dst[u]] = v[u];
                }
            }
            // ---- element-wise staging of the input window, zero outside X ----
            {
                const int total = p.ctch * p.plane;
                const int ih0 = h0 * g.sh - g.ph;
                for (int e0 = tid; e0 < total; e0 += 4 * kBlock) {
                    float v[4];
                    int dst[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int e = e0 + u * kBlock;
                        v[u] = 0.f; dst[u] = -1;
                        if (e < total) {
                            uint32_t c_l, rem, n_l, rem2, ih_l, iw_l;
                            p.d_plane.divmod(e, c_l, rem);
                            p.d_img.divmod(rem, n_l, rem2);
                            p.d_iwt.divmod(rem2, ih_l, iw_l);
                            const int c = c_first + c_l, n = n0 + n_l, ih = ih0 + (int)ih_l, iw = (int)iw_l - g.pw;
                            dst[u] = c_l * p.pp + rem;
                            if (c < g.C && n < g.N && ih >= 0 && ih < g.H && iw >= 0 && iw < g.W)
                                v[u] = load_elem<BF16>(p.X, (((long)n * g.C + c) * g.H + ih) * g.W + iw);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (dst[u] >= 0) Xs[dst[u]] = v[u];
                }
            }
            __syncthreads();
            contract();
        }
    }

    // ---- epilogue: every wavefront parks its accumulators in LDS in output order; then all
    //      threads add the WQ position slices and write rows of the result, coalesced ----
    __syncthreads();
    TRACE(9);
    {
        constexpr int RP = NCB + 1;                         // row pitch of the exchange buffer
        float *red = smem;                                  // [WQ][KT][RP]
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            int lo, lc;
            column_of<NT>(p, coltile, j, i16, c_first, lo, lc);
            if (lc < 0) lc = p.tap_mode ? (p.tile_c0[j] + i16) * RS + p.tile_tap[j] : j * 16 + i16;   // padding column: parked, never written out
#pragma unroll
            for (int v = 0; v < 4; ++v) red[(wq * KT + wk * 16 + 4 * kk + v) * RP + lc] = acc[j][v];
        }
        __syncthreads();
        TRACE(14);
        const int colbase = p.tap_mode ? c_first * RS : coltile * NCB;
        float *out = p.out + (long)split * g.K * CRS;
        for (int o = tid; o < KT * NCB; o += kBlock) {
            const int row = o / NCB, lc = o % NCB;
            float sum = red[row * RP + lc];
#pragma unroll
            for (int w = 1; w < WQ; ++w) sum += red[(w * KT + row) * RP + lc];
            const int k = k0 + row, col = colbase + lc;
            if (k < g.K && col < CRS) out[(long)k * CRS + col] = sum;
        }
    }
    TRACE(10);
}

// ------------------------------------------------------------------------------------
// Host side: tile plan and launch.
// ------------------------------------------------------------------------------------
#ifndef WGRAD_EXACT_KQ       // target number of staged dY elements (KT * Q) per tile
#define WGRAD_EXACT_KQ 8192
#endif
#ifndef WGRAD_EXACT_BLOCKS   // workgroups to aim for when splitting the reduction
#define WGRAD_EXACT_BLOCKS 512
#endif
constexpr size_t kMaxLds = 64 * 1024;

static int pitch_mod32(int len, int want, int multiple)
{
    // smallest pitch >= len with pitch % 32 == want (want is a multiple of `multiple`)
    int p = (len + multiple - 1) / multiple * multiple;
    while (p % 32 != want) p += multiple;
    return p;
}

static int largest_divisor_at_most(int n, int limit)
{
    if (limit >= n) return n;
    for (int d = limit; d >= 1; --d)
        if (n % d == 0) return d;
    return 1;
}

// Number of slices the reduction over positions is cut into, for a launch of nprob problems of
// this plan.  The baseline aims at a fixed number of workgroups.  The streaming form also weighs
// alternatives with a small model of a workgroup's life: a fixed cost (tables, first loads,
// epilogue), then its tiles one after another, each bounded by the matrix core shared with the
// other workgroups resident on the CU (as many as their LDS windows allow) plus a barrier's worth
// of skew; it matters for short reductions, where an uneven split (some workgroups with one tile
// more) or a second round of workgroups costs a large part of the whole.
int choose_splits(const ExactPlan &pl, int nprob, int want_blocks)
{
    const long tiles = (long)pl.h_tiles * pl.n_groups;
    const long out_tiles = (long)pl.ktiles * pl.ctiles * nprob;
    long base = ((want_blocks ? want_blocks : tune_int("WGRAD_EXACT_BLOCKS", WGRAD_EXACT_BLOCKS)) + out_tiles - 1) / out_tiles;
    if (base > tiles) base = tiles;
    if (base < 1) base = 1;
    if (want_blocks) {
        // a share of a mixed launch: the largest even cut not above the target
        long s = base;
        while (s > 1 && tiles % s != 0 && (tiles + s - 1) / s == (tiles + s - 2) / (s - 1)) --s;
        return (int)s;
    }
    // (layers with a handful of input channels are bound by their loads, not by the matrix core)
    if (!(pl.stream || pl.mm16) || pl.nt != 9 || !tune_int("WGRAD_EXACT_MODEL", 1)) return (int)base;

    int per_cu_max = (int)((size_t)160 * 1024 / (pl.lds_bytes ? pl.lds_bytes : 1));
    per_cu_max = per_cu_max > 4 ? 4 : (per_cu_max < 1 ? 1 : per_cu_max);
    if (pl.mm16 && per_cu_max > 2) per_cu_max = 2;                         // its registers allow two wavefronts per SIMD
    // us per tile and wavefront, loop efficiency included
    const double t_mfma = pl.mm16 ? 9.0 * 4 * pl.gpw * 16.0 / 2400.0 / 0.5 : pl.nt * 4.0 * pl.gpw * 32.0 / 2400.0 / 0.86;
    const double fixed = 9.0, skew = 0.5;                                  // skew: per resident workgroup
    auto cost = [&](long splits) {
        const long blocks = out_tiles * splits;
        const long rounds = (blocks + (long)kNumCU * per_cu_max - 1) / ((long)kNumCU * per_cu_max);
        // workgroups per CU: between the busiest CU and the average one (short launches behave like
        // the average, long ones like the busiest)
        double per_cu = 0.5 * ((blocks + kNumCU - 1) / kNumCU + (double)blocks / kNumCU);
        if (per_cu > per_cu_max) per_cu = per_cu_max;
        if (per_cu < 1) per_cu = 1;
        const long max_tiles = (tiles + splits - 1) / splits;
        return rounds * (fixed + max_tiles * per_cu * (t_mfma + skew)) + 0.002 * splits;   // slight preference for fewer partials
    };
    long best = base;
    double best_cost = cost(base) * 0.97;                                   // deviate only for a clear gain
    for (long s = 1; s <= tiles && s <= 1024; ++s) {
        const double c = cost(s);
        if (c < best_cost) { best_cost = c; best = s; }
    }
    return (int)best;
}

ExactPlan plan_exact(const Geometry &g, bool allow_stream)
{
    ExactPlan pl{};
    const int RS = g.R * g.S;
    const long CRS = g.crs();
    // (the rest of the plan is still made: tensors that are not 16-byte aligned take the general kernels)
    pl.plane2 = allow_stream && tune_int("WGRAD_EXACT_PLANE2", 1) && plane2_takes(g);
    pl.wk = g.K <= 16 ? 1 : (g.K <= 32 ? 2 : 4);
    const int KT = 16 * pl.wk, WQ = 4 / pl.wk;
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
    // the streaming form (A operand straight from global memory) takes every shape it can
    if (allow_stream && tune_int("WGRAD_EXACT_BF16MM", 1) && plan_exact_bf16(g, pl)) pl.ok = true;
    else if (allow_stream && tune_int("WGRAD_EXACT_STREAM", 1) && plan_exact_stream(g, pl)) pl.ok = true;

    // widest access the shape allows when staging X rows (alignment of the pointers is checked at launch)
    const int xv_shape = g.W % 4 == 0 ? 4 : (g.W % 2 == 0 ? 2 : 0);

    const int L = g.Ho * g.Wo;
    // pass 0 looks for the largest tile that fits LDS and the register pipeline of the vector
    // staging path (no ragged tiles: rows per tile divide Ho, images per tile divide N);
    // pass 1 (element-wise staging) only needs the tile to fit LDS
    for (int pass = 0; pass < 2 && !pl.ok; ++pass) {
        if (pass == 0 && (!xv_shape || L % 4 != 0)) continue;
        for (int qt = tune_int("WGRAD_EXACT_KQ", WGRAD_EXACT_KQ) / KT; qt >= 4; qt /= 2) {
            if (L >= qt) {
                pl.nti = 1;
                pl.ht = qt / g.Wo < 1 ? 1 : qt / g.Wo;
                pl.ht = pass == 0 ? largest_divisor_at_most(g.Ho, pl.ht) : (pl.ht > g.Ho ? g.Ho : pl.ht);
            } else {
                pl.ht = g.Ho;
                pl.nti = qt / L < 1 ? 1 : qt / L;
                pl.nti = pass == 0 ? largest_divisor_at_most(g.N, pl.nti) : (pl.nti > g.N ? g.N : pl.nti);
            }
            pl.q = pl.nti * pl.ht * g.Wo;
            pl.qpad = (pl.q + 8 * WQ - 1) / (8 * WQ) * (8 * WQ);    // an even number of 4-position steps per wavefront
            pl.qp = pitch_mod32(pl.qpad, 4, 4);
            pl.iht = (pl.ht - 1) * g.sh + g.R;
            pl.iwt = (g.Wo - 1) * g.sw + g.S;
            pl.pp = pitch_mod32(pl.nti * pl.iht * pl.iwt, 2, 1);
            size_t lds = ((size_t)KT * pl.qp + (size_t)pl.ctch * pl.pp + pl.qpad + 16) * 4;
            const size_t red = (size_t)4 * 16 * (pl.nt * 16 + 1) * 4;        // epilogue exchange buffer [WQ][KT][NT*16 + 1]
            if (red > lds) lds = red;
            pl.lds_bytes = lds;
            if (lds > kMaxLds) continue;
            pl.xv = 0;
            if (pass == 0) {
                const int seg = pl.ht * g.Wo;
                const long dy_slots = (long)KT * pl.nti * (seg / 4);
                const long x_slots = (long)pl.ctch * pl.nti * pl.iht * (g.W / xv_shape);
                const bool fits = seg % 4 == 0 && dy_slots <= slots_dy(pl.wk) * kBlock && x_slots <= slots_x(pl.wk) * kBlock
                                  && pl.iht <= 255 && (long)pl.ctch * pl.pp < (1 << 20)
                                  && (long)pl.nti * g.K * L < (1l << 31) && (long)pl.nti * g.C * g.H * g.W < (1l << 31);
                if (!fits) continue;
                pl.xv = xv_shape;
            }
            pl.ok = true;
            break;
        }
    }
    // fast-division bounds: dividend * divisor < 2^32
    const long plane = (long)pl.nti * pl.iht * pl.iwt;
    if (pl.ok && ((long)pl.ctch * plane * plane >= (1ll << 32) || (long)KT * pl.q * pl.q >= (1ll << 32))) pl.ok = false;
    if (!pl.ok || tune_int("WGRAD_EXACT_DIRECT", 0)) {
        // no tile of whole output rows fits (very wide or widely strided inputs): the general form
        plan_exact_direct(g, pl);
        return pl;
    }

    pl.h_tiles = (g.Ho + pl.ht - 1) / pl.ht;
    pl.n_groups = (g.N + pl.nti - 1) / pl.nti;
    pl.splits = choose_splits(pl, 1);
    pl.ws_bytes = pl.splits > 1 ? align_up((size_t)pl.splits * g.dw_elems() * 4) : 0;
    // tensors that are not 16-byte aligned fall back to the staged form at launch: size for both
    if (pl.stream || pl.mm16) {
        const size_t alt = plan_exact(g, false).ws_bytes;
        if (alt > pl.ws_bytes) pl.ws_bytes = alt;
    }
    return pl;
}

template <int NT, int WK, bool BF16, int XV>
static void launch_inst(const ExactParams &p, int grid, size_t lds, hipStream_t st)
{
    WGRAD_LAUNCH((wgrad_exact_mfma<NT, WK, BF16, XV>), dim3(grid), dim3(kBlock), lds, st, p);
}

template <int NT, int WK>
static void launch_dtype(const ExactParams &p, int grid, size_t lds, int xv, hipStream_t st)
{
    if (p.g.bf16) {
        if (xv == 4) launch_inst<NT, WK, true, 4>(p, grid, lds, st);
        else if (xv == 2) launch_inst<NT, WK, true, 2>(p, grid, lds, st);
        else launch_inst<NT, WK, true, 0>(p, grid, lds, st);
    } else {
        if (xv == 4) launch_inst<NT, WK, false, 4>(p, grid, lds, st);
        else if (xv == 2) launch_inst<NT, WK, false, 2>(p, grid, lds, st);
        else launch_inst<NT, WK, false, 0>(p, grid, lds, st);
    }
}

template <int NT>
static void launch_wk(const ExactParams &p, int wk, int grid, size_t lds, int xv, hipStream_t st)
{
    if (wk == 1) launch_dtype<NT, 1>(p, grid, lds, xv, st);
    else if (wk == 2) launch_dtype<NT, 2>(p, grid, lds, xv, st);
    else launch_dtype<NT, 4>(p, grid, lds, xv, st);
}

size_t exact_ws_per_problem(const Geometry &g, const ExactPlan &pl)
{
    (void)g;
    return pl.ws_bytes;
}

static bool batch_aligned(const Geometry &g, const Batch &b, int xv, int dyv)
{
    const int esz = g.bf16 ? 2 : 4;
    for (int i = 0; i < b.n; ++i)
        if (((uintptr_t)b.dY[i] % (dyv * esz)) != 0 || ((uintptr_t)b.X[i] % (xv * esz)) != 0) return false;
    return true;
}

static int launch_exact_staged(const Geometry &g, const ExactPlan &pl, const void *X, const void *dY, float *dW,
                               void *ws, hipStream_t st, CombineQueue *defer);

int launch_exact(const Geometry &g, const ExactPlan &plan, const Batch &b, void *ws, hipStream_t st, CombineQueue *defer,
                 MultiQueue *mq, int mq_blocks, Bf16Queue *bq)
{
    if (plan.plane2 && batch_aligned(g, b, 4, 4)) return launch_exact_plane2(g, b, st, mq);   // no split, no partial sums
    if (planes_bf16_takes(g) && batch_aligned(g, b, 8, 8)) return launch_exact_bf16_planes(g, b, st);   // likewise (bf16, 2x2 and 4x4 planes)
    if ((plan.stream || plan.mm16) && batch_aligned(g, b, plan.xv, plan.mm16 ? 8 : 4)) {
        // one launch for the whole batch; problem i owns the i-th slice of the workspace.  The
        // workgroup target is for the whole launch: a batch splits each reduction less finely.
        ExactPlan pl = plan;
        if (b.n > 1) {
            const int splits = choose_splits(pl, b.n);
            if (splits < pl.splits) pl.splits = splits;
        }
        if (mq && pl.stream && !g.bf16) {
            // part of a multi-shape launch: its workgroups share the chip with the other groups', so fewer
            // and longer ones do (a fixed cost per workgroup, less traffic in partial results)
            const int splits = choose_splits(pl, b.n, mq_blocks > 0 ? mq_blocks : 256);
            if (splits < pl.splits) pl.splits = splits;
        }
        if (bq && pl.mm16) {
            // one of several groups in a launch: the next group's workgroups fill the chip as this one's finish, so
            // half as many, twice as long, do -- half the partial results, and a workgroup's set-up and
            // write-out (a fifth of its life) paid half as often
            const int splits = choose_splits(pl, b.n, tune_int("WGRAD_BF16_MULTI_BLOCKS", 256));
            if (splits < pl.splits) pl.splits = splits;
        }
        float *out[kMaxBatch];
        const long prob_stride = (long)pl.splits * g.dw_elems();
        for (int i = 0; i < b.n; ++i) out[i] = pl.splits > 1 ? (float *)ws + i * prob_stride : b.dW[i];
        int rc = pl.mm16 ? launch_exact_bf16(g, pl, b, out, st, nullptr, bq) : launch_exact_stream(g, pl, b, out, st, mq);
        if (rc != WGRAD_OK) return rc;
        if (pl.splits > 1)
            return launch_combine((const float *)ws, prob_stride, pl.splits, g.dw_elems(), 1.0f, b.dW, b.n, st, defer);
        return WGRAD_OK;
    }
    // staged form: one problem at a time (shapes or alignments the streaming form does not take),
    // each in its own slice of the workspace
    const ExactPlan pl = (plan.stream || plan.mm16) ? plan_exact(g, false) : plan;
    for (int i = 0; i < b.n; ++i) {
        char *slice = (char *)ws + (size_t)i * align_up(plan.ws_bytes);
        if (pl.direct) {
            int rc = launch_exact_direct(g, pl, b.X[i], b.dY[i], b.dW[i], slice, st, defer);
            if (rc != WGRAD_OK) return rc;
            continue;
        }
        int rc = launch_exact_staged(g, pl, b.X[i], b.dY[i], b.dW[i], (char *)ws + (size_t)i * align_up(plan.ws_bytes), st, defer);
        if (rc != WGRAD_OK) return rc;
    }
    return WGRAD_OK;
}

static int launch_exact_staged(const Geometry &g, const ExactPlan &pl, const void *X, const void *dY, float *dW,
                               void *ws, hipStream_t st, CombineQueue *defer)
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
    // the vector staging path needs every access aligned: X to xv elements, dY to 4 elements
    const int esz = g.bf16 ? 2 : 4;
    int xv = pl.xv;
    if (xv && (((uintptr_t)dY % (4 * esz)) != 0 || ((uintptr_t)X % (xv * esz)) != 0)) xv = 0;
    const int dv = xv ? 4 : 1;
    p.d_segv = FastDiv(p.seg / dv);
    p.d_nsegv = FastDiv(pl.nti * (p.seg / dv));
    p.d_plane = FastDiv(p.plane);
    p.d_img = FastDiv(pl.iht * pl.iwt);
    p.d_iwt = FastDiv(pl.iwt);
    p.d_wv = FastDiv(xv ? g.W / xv : 1);
    p.d_rows = FastDiv(pl.nti * pl.iht);
    p.d_iht = FastDiv(pl.iht);
    p.d_rs = FastDiv(g.R * g.S);
    p.d_s = FastDiv(g.S);
    p.d_seg = FastDiv(p.seg);
    p.d_wo = FastDiv(g.Wo);
    p.d_htiles = FastDiv(pl.h_tiles);
    if (pl.tap_mode)
        for (int t = 0; t < pl.nt; ++t) {
            const int RS = g.R * g.S, tap = t % RS;
            p.tile_c0[t] = (t / RS) * 16;
            p.tile_toff[t] = (tap / g.S) * pl.iwt + tap % g.S;
            p.tile_tap[t] = tap;
        }

    const int grid = pl.ktiles * pl.ctiles * pl.splits;
    switch (pl.nt) {
        case 2: launch_wk<2>(p, pl.wk, grid, pl.lds_bytes, xv, st); break;
        case 4: launch_wk<4>(p, pl.wk, grid, pl.lds_bytes, xv, st); break;
        default: launch_wk<9>(p, pl.wk, grid, pl.lds_bytes, xv, st); break;
    }
    int rc = launch_status();
    if (rc != WGRAD_OK) return rc;
    if (pl.splits > 1) return launch_combine((const float *)ws, 0, pl.splits, g.dw_elems(), 1.0f, &dW, 1, st, defer);
    return WGRAD_OK;
}

}  // namespace wgrad
