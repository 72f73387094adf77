// Exact filter gradient, streaming form of the implicit GEMM (see exact_mfma.hip for the
// mathematics and the column mapping).  Differences from the staged form:
//
//   - dY, the A operand, never touches LDS.  MFMA 16x16x4 wants A[i][kk] from lane
//     (i = l%16, kk = l/16); the order of the reduction is free, so lane (i, kk) loads ONE
//     16-byte piece dY[k0+i][q0 + 4*kk .. +3] straight from global memory and feeds element
//     s of it to step s of a group of four steps.  (B must follow the same order: step s of
//     the group contracts positions q0 + 4*kk + s, kk = 0..3.)  A wavefront keeps one tile of
//     its A rows in registers (GPW pieces per lane); piece g of the next tile is requested
//     right after piece g of the current tile has been used, so the loads of a whole tile are
//     in flight behind the MFMAs.
//   - only the zero-haloed input window lives in LDS, double-buffered: the window of tile
//     t+1 is written (from registers loaded one tile earlier) at the start of tile t, so
//     there is a single barrier per tile.
//
// Every load is issued unconditionally (a lane or tile that has nothing to fetch re-reads
// the first element of a valid tile), which keeps the number of loads in flight fixed so a
// piece can be waited for while younger loads are still arriving.
#pragma once
#include "exact_common.hpp"

namespace wgrad {

// Instruction order inside one step of the MFMA pipeline (its region holds the LDS reads of
// step t+1 and the MFMAs of step t).  WGRAD_STREAM_SCHED = 2 (default): the reads are spread
// between the MFMAs (read, two MFMAs, read, two MFMAs, ...), so a wavefront never waits on an
// LDS read it has just issued; 1: all reads, then all MFMAs; 0: left to the compiler, which
// places each read right before its use.
#ifndef WGRAD_STREAM_SCHED
#define WGRAD_STREAM_SCHED 2
#endif
#if WGRAD_STREAM_SCHED == 1
#define WGRAD_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#else
#define WGRAD_SCHED_FENCE() do { } while (0)
#endif
#if WGRAD_STREAM_SCHED == 2
#define WGRAD_STEP_PATTERN(NT)                                                        \
    do {                                                                                \
        __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);   /* the address add      */ \
        for (int gsb = 0; gsb < (NT + 1) / 2; ++gsb) {                                  \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   /* one LDS read     */ \
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   /* two MFMAs        */ \
        }                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                              \
    } while (0)
#else
#define WGRAD_STEP_PATTERN(NT) do { } while (0)
#endif

// Everything a workgroup needs to know about its group but the tensors: in a launch that carries several groups the
// tensors of all of them sit in one table, so that nine groups fit the 4 KB of kernel arguments.
struct StreamShape {
    int per_prob;               // workgroups per problem
    Geometry g;
    int tap_mode, ktiles, ctiles, splits;
    int nti, ht, q, iht, iwt, pp, ctch, h_tiles, n_groups;
    int seg;                    // ht * Wo : contiguous dY elements per (image, channel) in a tile
    int xbuf;                   // floats per LDS window buffer (multiple of 4)
    int rowp;                   // LDS pitch of a window row (>= iwt)
    int wc;                     // column-uniform position order: 4-column blocks per output row (0: row-major order)
    int img4;                   // image-uniform position order on 4x4 planes (tiles of four whole images)
    int ipitch;                 // floats between the windows of consecutive images of a tile (iht * rowp, or more)
    FastDiv d_wv, d_rows, d_iht, d_rs, d_s, d_seg, d_wo, d_htiles;
    FastDiv d_gpi;              // column-uniform order: groups of 16 positions per image of a tile, (ht / 4) * wc
    int tile_c0[9], tile_toff[9], tile_tap[9];
};
struct StreamParams {
    const void *X[kMaxBatch], *dY[kMaxBatch];
    float *out[kMaxBatch];      // per problem: dW when splits == 1, else partials [splits][K][C*R*S]
    StreamShape s;
};

// Window staging slots (16- or 8-byte row pieces) per thread and tile.
__host__ __device__ constexpr int stream_xslots(int wk, int gpw)
{
    if (gpw == 2) return wk == 4 ? 3 : 5;
    return wk == 1 ? (gpw == 8 ? 9 : 5) : (wk == 2 ? (gpw == 8 ? 5 : 3) : (gpw == 8 ? 4 : 5));
}

// LDS offset (floats) of staged channel c_l.  In a step the four lane groups kk of an MFMA
// operand read positions 4 apart, so channels are placed such that
//   bank(c_l, kk) = (c_l & 3) + 8 * (c_l >> 2) + 4 * kk   (mod 32)
// is a bijection over 16 channels x 2 lane groups: pp = 1 (mod 32) is the pitch of a channel
// inside a quad, 4 * pp + 4 the pitch of a quad.
__device__ __forceinline__ int stream_chan_off(int c_l, int pp) { return (c_l & 3) * pp + (c_l >> 2) * (4 * pp + 4); }

template <int NT>
__device__ __forceinline__ void stream_column_of(const StreamShape &p, int coltile, int t, int i16, int c_first,
                                                 int &lds_off, int &local_col)
{
    const Geometry &g = p.g;
    const int RS = g.R * g.S;
    if (p.tap_mode) {
        const int c_l = p.tile_c0[t] + i16;
        const bool ok = c_first + c_l < g.C;
        lds_off = ok ? stream_chan_off(c_l, p.pp) + p.tile_toff[t] : 0;
        local_col = ok ? c_l * RS + p.tile_tap[t] : -1;
    } else {
        const int col = coltile * NT * 16 + t * 16 + i16;
        const bool ok = col < g.C * RS;
        uint32_t c, tap, r, s;
        p.d_rs.divmod(col, c, tap);
        p.d_s.divmod(tap, r, s);
        lds_off = ok ? (int)(stream_chan_off(c - c_first, p.pp) + r * p.iwt + s) : 0;
        local_col = ok ? t * 16 + i16 : -1;
    }
}

// NT: 16-column MFMA tiles per wavefront; WK: wavefronts along K; XV: elements per access
// when staging rows of X (4 or 2); GPW: 16-position groups per wavefront and tile (a tile
// has 16 * GPW * (4/WK) positions, padded with zero positions if the shape gives fewer).
// ROWP: for 3x3 filters in tap mode, the LDS pitch of a window row as a compile-time constant:
// the nine taps of a step are then one per-lane address plus nine immediate offsets, and the
// loop has one VALU instruction per nine MFMAs instead of nine (the adds, not LDS or the matrix
// core, bound the loop otherwise).  ROWP = 0: run-time pitch and tap offsets (any filter).
// WC (3x3, stride 1, padding 1, output rows of 4 * WC positions, tiles of a multiple of four rows): the
// positions of a tile are taken in column-uniform order -- a group of 16 is four rows x four columns, lane group
// kk holding row kk of it -- so that the four positions an MFMA step contracts share their column.  A step on the
// first (last) column of a row then multiplies the taps of filter column 0 (2) with the zero halo only: those
// three MFMAs and their LDS reads are left out, statically (the step's column block is gi % WC).  That is 1/6 of
// the matrix work on 4x4 planes, 1/12 on 8x8.  WC = 0: row-major order, every tap multiplied.
// IMG4 (4x4 planes, tiles of eight images, eight groups per wavefront): image-uniform order -- group gi is output
// row gi % 4 of the four images 4 * (gi / 4) .. + 3, lane group kk holding image kk's row -- so the four positions
// of a step are ONE position (gi % 4, st) of four images and every tap that falls outside X for that position, by
// row or by column, is left out: 100 of a plane's 144 (position, tap) pairs remain, exactly the products that do
// not multiply padding.
// The body takes the workgroup's number `bid` among the `nblk` workgroups of its launch (or of its
// share of a launch that carries several shapes) and the dynamic LDS.
template <int NT, int WK, bool BF16, int XV, int GPW, int ROWP, int WC = 0, bool IMG4 = false>
__device__ __forceinline__ void stream_body(const StreamShape &p, const void *const *Xt, const void *const *dYt, float *const *outt,
                                            float *smem, int bid, int nblk)
{
    static_assert(ROWP == 0 || NT == 9, "immediate tap offsets are for 3x3 filters in tap mode");
    static_assert(!IMG4 || (WC == 1 && GPW % 4 == 0 && WK == 4), "the image-uniform order is for 4x4 planes: four images = four groups, one per output row");
    static_assert(WC == 0 || (ROWP != 0 && GPW % WC == 0), "the column-uniform order needs immediate taps and whole rows of blocks per wavefront");
    const int rowp = ROWP ? ROWP : p.rowp;
    constexpr int KT = 16 * WK, WQ = 4 / WK;
    constexpr int ESZ = BF16 ? 2 : 4;
    constexpr int NCB = NT * 16;
    constexpr int QT = 16 * GPW * WQ;                   // positions per tile, padded
    constexpr int XS = stream_xslots(WK, GPW);
    float *Xs0 = smem;                                  // [2][xbuf]
    int *xoff = (int *)(smem + 2 * p.xbuf);             // [QT] byte offsets

    const Geometry &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wk = wave % WK, wq = wave / WK;
    const int i16 = lane & 15, kk = lane >> 4;
    const int RS = g.R * g.S, CRS = g.C * RS;
    const int L = g.Ho * g.Wo;

    // a launch may carry several problems of identical shape (layers of a schedule run)
    const int logical_all = xcd_contiguous_id(bid, nblk);
    const int prob = logical_all / p.per_prob;
    const int logical = logical_all - prob * p.per_prob;
    const char *const Xp = (const char *)Xt[prob];
    const char *const dYp = (const char *)dYt[prob];
    const int coltile = logical % p.ctiles;
    const int ktile = (logical / p.ctiles) % p.ktiles;
    const int split = logical / (p.ctiles * p.ktiles);
    const int k0 = ktile * KT;
    const int c_first = p.tap_mode ? coltile * 16 * (NT / RS) : (coltile * NT * 16) / RS;

    TRACE(0);
    TRACE_BLK(0);
    float4_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int tiles_total = p.h_tiles * p.n_groups;
    const int wt_begin = (int)((long)split * tiles_total / p.splits);
    const int wt_end = (int)((long)(split + 1) * tiles_total / p.splits);

    // ---- A operand: this lane's pieces of a tile, as byte offsets from the tile's first element ----
    const int k_row = k0 + wk * 16 + i16;
    uint32_t a_off[GPW];
    uint32_t a_live = 0;                                // bit g: piece g holds real data for this lane
#pragma unroll
    for (int gi = 0; gi < GPW; ++gi) {
        const int q = 16 * (wq * GPW + gi) + 4 * kk;
        a_off[gi] = 0;
        if (q < p.q && k_row < g.K) {
            uint32_t n_l, rem;
            if (IMG4) {                     // group = (four images, output row), lane group = image
                n_l = 4 * ((wq * GPW + gi) >> 2) + kk;
                rem = 4 * ((wq * GPW + gi) & 3);
            } else if (WC) {                // group -> (image, block of four rows, block of four columns); kk = row in the block
                uint32_t gimg;
                p.d_gpi.divmod((uint32_t)(wq * GPW + gi), n_l, gimg);
                rem = (4 * (gimg / WC) + kk) * g.Wo + 4 * (gimg % WC);
            } else {
                p.d_seg.divmod(q, n_l, rem);
            }
            a_off[gi] = ((n_l * g.K + (wk * 16 + i16)) * L + rem) * ESZ;
            a_live |= 1u << gi;
        }
    }
    TRACE(19);
    // ---- X window: this thread's staging slots (row pieces), decoded once ----
    int x_pack[XS];              // LDS float index | ih_l << 20 | valid elements << 28, -1 = unused
    uint32_t x_src[XS];          // byte offset from row 0 of the tile's first (image, channel)
    {
        const int x_total = p.ctch * p.nti * p.iht * (int)p.d_wv.d;
#pragma unroll
        for (int u = 0; u < XS; ++u) {
            const int e = tid + u * kBlock;
            x_pack[u] = -1; x_src[u] = 0;
            if (e < x_total) {
                uint32_t row, jv, c_l, rem, n_l, ih_l;
                p.d_wv.divmod(e, row, jv);
                p.d_rows.divmod(row, c_l, rem);
                p.d_iht.divmod(rem, n_l, ih_l);
                const int col0 = g.pw + jv * XV;             // window column of the first element
                int nv = p.iwt - col0;                       // columns right of the window are not staged
                nv = nv > XV ? XV : nv;
                if (c_first + (int)c_l < g.C && nv > 0) {
                    x_pack[u] = (int)(stream_chan_off(c_l, p.pp) + n_l * p.ipitch + ih_l * rowp + col0) | (int)(ih_l << 20) | (nv << 28);
                    x_src[u] = ((n_l * g.C + c_l) * (g.H * g.W) + jv * XV) * ESZ;
                }
            }
        }
    }
    TRACE(1);

    Vec<BF16, 4> ring[GPW];
    Vec<BF16, XV> xr[XS];
    uint32_t x_row_ok = 0;

    // tile wt (or, past the end, a dummy re-read of the first element of the last tile)
    auto tile_origin = [&](int wt, bool live, const char *&dy_base, const char *&x_base, int &ih0) {
        const int w = live ? wt : wt_end - 1;
        uint32_t ng, hti;
        p.d_htiles.divmod(w, ng, hti);
        const int n0 = ng * p.nti, h0 = hti * p.ht;
        dy_base = dYp + (((long)n0 * g.K + k0) * g.Ho + h0) * g.Wo * ESZ;
        x_base = Xp + ((long)n0 * g.C + c_first) * g.H * g.W * ESZ;
        ih0 = h0 * g.sh - g.ph;
    };
    auto load_x = [&](int wt) {
        const bool live = wt < wt_end;
        const char *dyb, *xb;
        int ih0;
        tile_origin(wt, live, dyb, xb, ih0);
        x_row_ok = 0;
#pragma unroll
        for (int u = 0; u < XS; ++u) {
            int ih = ih0 + ((x_pack[u] >> 20) & 0xff);
            if (ih >= 0 && ih < g.H) x_row_ok |= 1u << u;
            ih = ih < 0 ? 0 : (ih >= g.H ? g.H - 1 : ih);
            xr[u].load(xb, live ? x_src[u] + ih * (g.W * ESZ) : 0u);
        }
    };
    auto commit_x = [&](float *buf) {
#pragma unroll
        for (int u = 0; u < XS; ++u)
            if (x_pack[u] >= 0) {
                float *dst = buf + (x_pack[u] & 0xfffff);
                const int nv = x_pack[u] >> 28;
                const bool ok = (x_row_ok >> u) & 1;
#pragma unroll
                for (int i = 0; i < XV; ++i)
                    if (i < nv) dst[i] = ok ? xr[u].get(i) : 0.f;
            }
    };

    // ---- prologue: window and A pieces of the first tile, window registers of the second ----
    {
        const char *dyb, *xb;
        int ih0;
        load_x(wt_begin);
        tile_origin(wt_begin, true, dyb, xb, ih0);
#pragma unroll
        for (int gi = 0; gi < GPW; ++gi) ring[gi].load(dyb, a_off[gi]);
        TRACE(20);
    }
    // ---- LDS tables and the zero fill, while the first loads are in flight ----
    int coloff[NT];                                     // byte offsets into a window buffer
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int lc;
        stream_column_of<NT>(p, coltile, t, i16, c_first, coloff[t], lc);
        coloff[t] *= 4;
    }
    // ROWP != 0: one channel per lane; the taps are immediates (a padding channel reads channel 0, unused)
    const int lane_base = (c_first + i16 < g.C ? stream_chan_off(i16, p.pp) : 0) * 4;
    auto read_b = [&](const char *Xw, int xo, float (&b)[NT]) {
        if (ROWP) {
            const float *q = (const float *)(Xw + lane_base + xo);
#pragma unroll
            for (int j = 0; j < NT; ++j) b[j] = q[(j / 3) * ROWP + j % 3];
        } else {
#pragma unroll
            for (int j = 0; j < NT; ++j) b[j] = *(const float *)(Xw + coloff[j] + xo);
        }
    };
    TRACE(16);
    // byte offset of staged position q inside a staged input channel; padded positions read offset 0
    for (int q = tid; q < QT; q += kBlock) {
        int off = 0;
        if (q < p.q) {
            uint32_t n_l, rem, h_l, w;
            if (IMG4) {
                n_l = 4 * (q >> 6) + ((q >> 2) & 3); h_l = (q >> 4) & 3; w = q & 3;
            } else if (WC) {
                uint32_t gimg;
                p.d_gpi.divmod((uint32_t)q >> 4, n_l, gimg);
                h_l = 4 * (gimg / WC) + ((q >> 2) & 3);
                w = 4 * (gimg % WC) + (q & 3);
            } else {
                p.d_seg.divmod(q, n_l, rem);
                p.d_wo.divmod(rem, h_l, w);
            }
            off = (n_l * p.ipitch + h_l * g.sh * rowp + w * g.sw) * 4;
        }
        xoff[q] = off;
    }
    TRACE(17);
    // staging writes only cells that hold data: halo columns and unused channels stay zero
    for (int e = tid; e < (2 * p.xbuf) >> 2; e += kBlock) ((float4_t *)smem)[e] = float4_t{0.f, 0.f, 0.f, 0.f};

    TRACE(18);
    {
        __syncthreads();                      // zero fill and tables complete
        TRACE(21);
        commit_x(Xs0);
        TRACE(22);
        load_x(wt_begin + 1);
#ifndef WGRAD_STREAM_NOSETTLE
        // Enter the loop with no load pending.  The memory counter is in-order and the compiler merges what is
        // pending on the entry path with what is pending around the loop: in the loop the window pieces are
        // older than the operand pieces requested after them and the commit may leave those in flight; on the
        // entry path they are the youngest loads.  Merged, every tile would begin by waiting for everything,
        // the operand pieces requested late in the tile before included.
#pragma unroll
        for (int u = 0; u < XS; ++u) xr[u].settle();
#pragma unroll
        for (int gi = 0; gi < GPW; ++gi) ring[gi].settle();
#endif
    }
    TRACE(2);

    const int xo_base = 16 * wq * GPW + 4 * kk;           // this lane's first position in a tile
    int par = 0;
    for (int wt = wt_begin; wt < wt_end; ++wt, par ^= 1) {
        __syncthreads();   // window of tile wt is complete; everyone has left the buffer tile wt+1 goes to
        if (wt == wt_begin) TRACE(3);
        if (wt == wt_begin + 1) TRACE(5);
        const char *Xw = (const char *)(Xs0 + par * p.xbuf);
        // window of the next tile: registers -> the other buffer, then request the one after it
        commit_x(Xs0 + (par ^ 1) * p.xbuf);
        if (wt == wt_begin + 1) TRACE(6);
        load_x(wt + 2);
        const bool has_next = wt + 1 < wt_end;
        const char *dyb, *xb;
        int ih0;
        tile_origin(wt + 1, has_next, dyb, xb, ih0);
        if (wt == wt_begin + 1) TRACE(7);

        {
            // The 4 * GPW steps of the tile form one software pipeline: the LDS reads of step t+1
            // (and the position offsets of the next group) are issued before the MFMAs of step t,
            // across group boundaries too.  Everything below is unrolled; indices are constants.
            constexpr int T = 4 * GPW;
            float bq[2][NT];
            float a_cur[4];
            int4 xo_cur = *(const int4 *)(xoff + xo_base), xo_nxt = xo_cur;
            {
                const bool live = a_live & 1u;
#pragma unroll
                for (int e = 0; e < 4; ++e) a_cur[e] = live ? ring[0].get(e) : 0.f;
                ring[0].load(dyb, has_next ? a_off[0] : 0u);      // piece 0 of the next tile
            }
            read_b(Xw, xo_cur.x, bq[0]);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const int gi = t >> 2, st = t & 3;
                if (st == 0 && gi + 1 < GPW) xo_nxt = *(const int4 *)(xoff + xo_base + 16 * (gi + 1));
                if (t + 1 < T) {
                    const int xo = st == 0 ? xo_cur.y : (st == 1 ? xo_cur.z : (st == 2 ? xo_cur.w : xo_nxt.x));
                    read_b(Xw, xo, bq[(t + 1) & 1]);
                }
                WGRAD_SCHED_FENCE();
                // column-uniform order: this step's four positions lie on column 4 * (gi % WC) + st of their rows
                const bool first_col = WC && st == 0 && gi % (WC ? WC : 1) == 0;
                const bool last_col = WC && st == 3 && gi % (WC ? WC : 1) == (WC ? WC : 1) - 1;
                // image-uniform order: the step is output row gi of its four images
                const bool first_row = IMG4 && gi % 4 == 0, last_row = IMG4 && gi % 4 == 3;
#pragma unroll
                for (int j = 0; j < NT; ++j) {
                    if ((first_col && j % 3 == 0) || (last_col && j % 3 == 2)) continue;      // taps on the zero halo
                    if ((first_row && j / 3 == 0) || (last_row && j / 3 == 2)) continue;
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[st], bq[t & 1][j], acc[j], 0, 0, 0);
                }
                WGRAD_SCHED_FENCE();
                WGRAD_STEP_PATTERN(NT);
                if (st == 3 && gi + 1 < GPW) {
                    // next group: its A piece leaves the ring (which is refilled for the next tile)
                    xo_cur = xo_nxt;
                    const bool live = (a_live >> (gi + 1)) & 1u;
#pragma unroll
                    for (int e = 0; e < 4; ++e) a_cur[e] = live ? ring[gi + 1].get(e) : 0.f;
                    ring[gi + 1].load(dyb, has_next ? a_off[gi + 1] : 0u);
                }
            }
        }
        if (wt == wt_begin) TRACE(4);
        if (wt == wt_begin + 1) TRACE(11);
    }
    TRACE(8);

    // ---- epilogue: every wavefront parks its accumulators in LDS, column-major with the four rows a
    //      lane holds side by side (one 16-byte write per column tile); then all threads add the WQ
    //      position slices, four rows at a time, and write rows of the result, coalesced ----
    __syncthreads();
    TRACE(9);
    {
        constexpr int KTP = KT + 4;                         // floats per parked column (16-byte multiple, odd in units of 16 bytes)
        float *red = smem;                                  // [WQ][NCB][KTP]
#pragma unroll
        for (int j = 0; j < NT; ++j) {
            int lo, lc;
            stream_column_of<NT>(p, coltile, j, i16, c_first, lo, lc);
            if (lc < 0) lc = p.tap_mode ? (p.tile_c0[j] + i16) * RS + p.tile_tap[j] : j * 16 + i16;   // padding column: parked, never written out
            *(float4_t *)(red + ((wq * NCB + lc) * KTP + wk * 16 + 4 * kk)) = acc[j];
        }
        __syncthreads();
        TRACE(14);
        const int colbase = p.tap_mode ? c_first * RS : coltile * NCB;
        float *out = outt[prob] + (long)split * g.K * CRS;
        for (int o = tid; o < (KT / 4) * NCB; o += kBlock) {
            const int rq = o / NCB, lc = o % NCB;
            float4_t sum = *(const float4_t *)(red + (lc * KTP + 4 * rq));
#pragma unroll
            for (int w = 1; w < WQ; ++w) sum += *(const float4_t *)(red + ((w * NCB + lc) * KTP + 4 * rq));
            const int col = colbase + lc;
            if (col < CRS) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int k = k0 + 4 * rq + v;
                    if (k < g.K) out[(long)k * CRS + col] = sum[v];
                }
            }
        }
    }
    TRACE(10);
    TRACE_BLK(1);
}

template <int NT, int WK, bool BF16, int XV, int GPW, int ROWP, int WC = 0, bool IMG4 = false>
__global__ __launch_bounds__(kBlock) void wgrad_exact_stream(const StreamParams p)
{
    extern __shared__ float smem[];
    stream_body<NT, WK, BF16, XV, GPW, ROWP, WC, IMG4>(p.s, p.X, p.dY, p.out, smem, blockIdx.x, gridDim.x);
}

// A prepared launch of the streaming kernel, and a queue of them for a multi-shape launch.
constexpr int kMultiMax = 9;        // groups per multi-shape launch (their parameters are kernel arguments)
constexpr int kMultiTensors = 24;   // layers per multi-shape launch (their tensors are one table in the kernel arguments)
struct StreamLaunch {
    StreamParams p;
    int nt, wk, xv, gpw, rowp_inst, wc, img4, grid;
    int plane2;                 // the 2x2-plane matrix-product form (exact_plane2_kernel.hpp): only the tensors, g and per_prob of p are set
    int nprob;                  // problems (layers) of the group
    size_t lds;
};
struct MultiQueue {
    int n = 0;
    int tensors = 0;            // problems of the queued groups
    StreamLaunch item[kMultiMax];
};
int multi_variant(int nt, int wk, int xv, int gpw, int rowp, int wc, int img4);     // -1: not among the shapes a multi launch mixes
int launch_stream_now(const StreamLaunch &L, hipStream_t st);
void launch_plane2_kernel(const StreamLaunch &L, hipStream_t st);
int multi_flush(MultiQueue &q, hipStream_t st);

// Per-K-tile-width launchers, each instantiated in its own translation unit.
void stream_launch_w1(const StreamParams &p, int nt, int xv, int gpw, int rowp, int grid, size_t lds, hipStream_t st);
void stream_launch_w2(const StreamParams &p, int nt, int xv, int gpw, int rowp, int grid, size_t lds, hipStream_t st);
void stream_launch_w4(const StreamParams &p, int nt, int xv, int gpw, int rowp, int grid, size_t lds, hipStream_t st);

// The column-uniform instantiations (WC blocks of four columns per output row).
template <int WK, int GPW, int ROWP, int WC, bool IMG4 = false>
static void stream_inst_wc(const StreamParams &p, int grid, size_t lds, hipStream_t st)
{
    WGRAD_LAUNCH((wgrad_exact_stream<9, WK, false, 4, GPW, ROWP, WC, IMG4>), dim3(grid), dim3(kBlock), lds, st, p);
}

template <int NT, int WK, bool BF16, int XV, int ROWP>
static void stream_inst(const StreamParams &p, int gpw, int grid, size_t lds, hipStream_t st)
{
    // more than 64 KB of dynamic LDS has to be granted per kernel function (the CU has 160 KB)
    if (gpw == 8) {
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)wgrad_exact_stream<NT, WK, BF16, XV, 8, ROWP>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return;
        WGRAD_LAUNCH((wgrad_exact_stream<NT, WK, BF16, XV, 8, ROWP>), dim3(grid), dim3(kBlock), lds, st, p);
    } else if (gpw == 4) {
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)wgrad_exact_stream<NT, WK, BF16, XV, 4, ROWP>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return;
        WGRAD_LAUNCH((wgrad_exact_stream<NT, WK, BF16, XV, 4, ROWP>), dim3(grid), dim3(kBlock), lds, st, p);
    } else {
        // short tiles: strided layers, whose input window is four times the size of the output tile
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)wgrad_exact_stream<NT, WK, BF16, XV, 2, ROWP>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return;
        WGRAD_LAUNCH((wgrad_exact_stream<NT, WK, BF16, XV, 2, ROWP>), dim3(grid), dim3(kBlock), lds, st, p);
    }
}

template <int WK, bool BF16>
static void stream_pick(const StreamParams &p, int nt, int xv, int gpw, int rowp, int grid, size_t lds, hipStream_t st)
{
    if (nt == 9) {
        if constexpr (WK == 4 && !BF16) {
            if (p.s.wc == 1 && p.s.img4 && rowp == 6 && xv == 4 && gpw == 8) { stream_inst_wc<4, 8, 6, 1, true>(p, grid, lds, st); return; }
            if (p.s.wc == 1 && rowp == 12 && xv == 4 && gpw == 4) { stream_inst_wc<4, 4, 12, 1>(p, grid, lds, st); return; }
            if (p.s.wc == 2 && rowp == 12 && xv == 4 && gpw == 8) { stream_inst_wc<4, 8, 12, 2>(p, grid, lds, st); return; }
            if (p.s.wc == 4 && rowp == 20 && xv == 4 && gpw == 8) { stream_inst_wc<4, 8, 20, 4>(p, grid, lds, st); return; }
            if (p.s.wc == 8 && rowp == 36 && xv == 4 && gpw == 8) { stream_inst_wc<4, 8, 36, 8>(p, grid, lds, st); return; }
        }
        if constexpr (WK == 2 && !BF16) {
            if (p.s.wc == 4 && rowp == 20 && xv == 4 && gpw == 8) { stream_inst_wc<2, 8, 20, 4>(p, grid, lds, st); return; }
        }
        if (rowp == 4 && xv == 2) stream_inst<9, WK, BF16, 2, 4>(p, gpw, grid, lds, st);
        else if (rowp == 12 && xv == 4) stream_inst<9, WK, BF16, 4, 12>(p, gpw, grid, lds, st);
        else if (rowp == 20 && xv == 4) stream_inst<9, WK, BF16, 4, 20>(p, gpw, grid, lds, st);
        else if (rowp == 36 && xv == 4) stream_inst<9, WK, BF16, 4, 36>(p, gpw, grid, lds, st);
        else if (xv == 4) stream_inst<9, WK, BF16, 4, 0>(p, gpw, grid, lds, st);
        else stream_inst<9, WK, BF16, 2, 0>(p, gpw, grid, lds, st);
    } else if (nt == 4) {
        if (xv == 4) stream_inst<4, WK, BF16, 4, 0>(p, gpw, grid, lds, st);
        else stream_inst<4, WK, BF16, 2, 0>(p, gpw, grid, lds, st);
    } else {
        if (xv == 4) stream_inst<2, WK, BF16, 4, 0>(p, gpw, grid, lds, st);
        else stream_inst<2, WK, BF16, 2, 0>(p, gpw, grid, lds, st);
    }
}

// pairs (rowp, xv) that have an immediate-offset instantiation
inline bool stream_has_rowp(int rowp, int xv) { return (rowp == 4 && xv == 2) || ((rowp == 6 || rowp == 12 || rowp == 20 || rowp == 36) && xv == 4); }

}  // namespace wgrad
