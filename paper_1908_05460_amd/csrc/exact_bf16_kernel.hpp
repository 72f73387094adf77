// Exact filter gradient for bf16 inputs on the bf16 matrix core (v_mfma_f32_16x16x32_bf16, fp32
// accumulate): the streaming implicit GEMM of exact_stream_kernel.hpp re-cut for an instruction
// that contracts 32 positions at once.  3x3 filters, stride 1, padding 1, C a multiple of 16 and
// K a multiple of 64; everything else stays on the fp32 matrix-core kernels.
//
//   - A operand (dY): lane (i = l%16, kk = l/16) of the instruction holds row i, reduction slots
//     8kk..8kk+7.  The order of the reduction is free, so the slots of a 32-position group are the
//     positions themselves: the lane loads the 16 bytes dY[k][q0+8kk .. +7] straight from global
//     memory and that register quadruple IS the operand.  A wavefront owns MT = 4 row tiles
//     (64 output channels), so a B operand read from LDS feeds four instructions.
//   - B operand (X): lane (c = l%16, kk) needs the eight input elements that positions
//     q0+8kk..+7 see through tap (r,s).  The window is kept in LDS as bf16, row-major with a
//     zero halo, and positions are handled in pairs (w, w+1), w even: for a window row the lane
//     reads, per pair, the two aligned 32-bit words that hold columns w..w+3; the word of tap
//     s = 0 is the first, of s = 2 the second, of s = 1 their middle (one v_alignbit).  One read
//     per pair and row therefore serves the three taps of that row: 12 two-word reads per 36
//     matrix instructions.
//   - Pipeline, tiles, splits, workgroup numbering: as in the fp32 streaming kernel (window
//     double-buffered, one barrier per tile, every load unconditional).
#pragma once
#include "exact_common.hpp"

namespace wgrad {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

struct Bf16Params {
    const void *X[kMaxBatch], *dY[kMaxBatch];
    float *out[kMaxBatch];      // per problem: dW when splits == 1, else partials [splits][K][C*9]
    const int32_t *hw[kMaxBatch];   // SPARSE: selected position of every map, (row << 16 | col), [N][K]
    const float *sum[kMaxBatch];    // SPARSE: sum of every map, [N][K]
    float scale;                // applied to what the kernel writes
    int per_prob;               // workgroups per problem
    Geometry g;
    int ktiles, ctiles, splits;
    int nti, ht, q, iht, h_tiles, n_groups;
    int seg;                    // ht * Wo : contiguous dY elements per (image, channel) in a tile
    int ppw;                    // 32-bit words between the planes of a channel quad (1 mod 32)
    int buf_words;              // words per window buffer
    int rowp;                   // elements per window row (even)
    FastDiv d_wv, d_rows, d_iht, d_seg, d_wo, d_htiles;
};

constexpr int kBf16MT = 4;      // 16-row tiles per wavefront
constexpr int kBf16KT = 16 * kBf16MT;

// Word offset of staged channel c_l inside a window copy.  The four lane groups of an operand read
// words 4 apart (8 positions), so with ppw = 1 (mod 32)
//   bank(c_l, kk) = (c_l & 3) + 16 * ((c_l >> 2) & 1) + 4 * kk   (mod 32)
// takes every value exactly twice over 16 channels x 4 groups: the minimum for 64 lanes.
__host__ __device__ __forceinline__ int bf16_chan_off(int c_l, int ppw) { return (c_l & 3) * ppw + (c_l >> 2) * (4 * ppw + 12); }

// Elements of a window staging piece: 16-byte pieces where the input rows are a multiple of eight long
// (the row pitches 12, 20, 36 belong to rows of 8, 16, 32), 8-byte pieces otherwise.
__host__ __device__ constexpr int bf16_xv(int rowp) { return rowp >= 12 ? 8 : 4; }
// Window staging slots (pieces) per thread and tile.
__host__ __device__ constexpr int bf16_xslots(int gpw, int rowp) { return rowp >= 12 ? 3 : (gpw >= 2 ? 5 : 3); }

// GPW: 32-position groups per wavefront and tile (the four wavefronts split the positions of a
// tile, 128 * GPW in all, padded with dead positions if the shape gives fewer).
// ROWP: window row pitch in elements, compile-time so that the tap offsets are immediates.
// FULL: every position of a tile is a real one (q == 128 * GPW): the A registers are then used as
// loaded; otherwise the pieces of dead positions are replaced by zeros first.
// SPARSE: the A operand is not dY but the sparsified gradient of the max-gradient approximation
// (Section 2.4: its filter gradient is the exact one of a dY that keeps one entry per map): a map
// is given by its selected position and its sum, and a lane builds its operand in registers -- the
// sum, rounded to bf16, in the slot of the selected position if that is one of its eight, zeros
// elsewhere.  Nothing of dY is read.
// P4: 2x2 planes (H = W = 2).  A map is four elements, so a lane's eight positions are two images
// (two 8-byte loads of dY), and an input plane is staged whole: one 8-byte piece per (image, channel).
// The body takes the workgroup's number `bid` among the `nblk` workgroups of its launch (or of its group in
// a launch that carries several shapes) and the dynamic LDS.
template <int GPW, int ROWP, bool FULL, bool P4, bool SPARSE>
__device__ __forceinline__ void bf16_body(const Bf16Params &p, float *smem, int bid, int nblk)
{
    constexpr int MT = kBf16MT, KT = kBf16KT, NT = 9, NCB = NT * 16;
    constexpr bool ROW8 = ROWP >= 12;                   // map rows of 8, 16 or 32: a lane's eight positions share a row
    constexpr int QT = 128 * GPW;
    constexpr int XS = bf16_xslots(GPW, ROWP), XV = bf16_xv(ROWP);
    uint32_t *Xs0 = (uint32_t *)smem;                   // [2][buf_words]
    int *xoffp = (int *)(Xs0 + 2 * p.buf_words);        // [QT / 2] byte offsets of position pairs

    const Geometry &g = p.g;
    const int tid = threadIdx.x, lane = tid & 63, wq = tid >> 6;
    const int i16 = lane & 15, kk = lane >> 4;
    const int L = g.Ho * g.Wo, CRS = g.C * 9;

    const int logical_all = xcd_contiguous_id(bid, nblk);
    const int prob = logical_all / p.per_prob;
    const int logical = logical_all - prob * p.per_prob;
    const char *const Xp = (const char *)p.X[prob];
    const char *const dYp = SPARSE ? (const char *)p.hw[prob] : (const char *)p.dY[prob];
    const char *const sump = (const char *)p.sum[prob];
    const int coltile = logical % p.ctiles;
    const int ktile = (logical / p.ctiles) % p.ktiles;
    const int split = logical / (p.ctiles * p.ktiles);
    const int k0 = ktile * KT;
    const int c_first = coltile * 16;

    TRACE(0);
    TRACE_BLK(0);
    float4_t acc[MT][NT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[m][t] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int tiles_total = p.h_tiles * p.n_groups;
    const int wt_begin = (int)((long)split * tiles_total / p.splits);
    const int wt_end = (int)((long)(split + 1) * tiles_total / p.splits);

    // First of the eight positions this lane contracts in group gi.  Groups come in pairs whose lanes
    // take adjacent runs of eight positions, so that the two 16-byte pieces a lane loads for a pair
    // share a 128-byte line with the other three lanes of its row.
    auto first_position = [&](int gi) {
        return GPW % 2 == 0 ? 64 * (wq * (GPW / 2) + gi / 2) + 16 * kk + 8 * (gi & 1) : 32 * (wq * GPW + gi) + 8 * kk;
    };
    // ---- A operand: byte offsets of this lane's 16-byte pieces from the tile's first element ----
    uint32_t a_off[GPW];
    int a_pos[GPW];                                     // SPARSE: position within the tile's rows of the lane's first slot
    uint32_t a_live = 0;
#pragma unroll
    for (int gi = 0; gi < GPW; ++gi) {
        const int q = first_position(gi);
        a_off[gi] = 0; a_pos[gi] = 0;
        if (q < p.q) {
            uint32_t n_l, rem;
            p.d_seg.divmod(q, n_l, rem);
            a_off[gi] = SPARSE ? (n_l * g.K + i16) * 4 : ((n_l * g.K + i16) * L + rem) * 2;
            a_pos[gi] = rem;
            a_live |= 1u << gi;
        }
    }
    const uint32_t row_tile_bytes = SPARSE ? 64u : 16u * L * 2u;       // from row tile m to m + 1
    const uint32_t image_bytes = SPARSE ? (uint32_t)g.K * 4u : (uint32_t)g.K * L * 2u;  // P4: to the same channel's map of the next image
    // uniform base + 32-bit lane offset: the address needs no vector arithmetic
    auto load_a = [&](const char *base, uint32_t off) -> uint4_t {
        if (SPARSE) {
            // (position, sum) of the lane's map, and of the next image's for 2x2 planes
            const char *sbase = sump + (base - dYp);
            uint4_t v{*(const uint32_t *)(base + off), *(const uint32_t *)(sbase + off), 0u, 0u};
            if (P4) { v[2] = *(const uint32_t *)(base + image_bytes + off); v[3] = *(const uint32_t *)(sbase + image_bytes + off); }
            return v;
        }
        if (P4) {
            const uint2 lo = *(const uint2 *)(base + off), hi = *(const uint2 *)(base + image_bytes + off);
            return uint4_t{lo.x, lo.y, hi.x, hi.y};
        }
        return *(const uint4_t *)(base + off);
    };

    // ---- X window: this thread's staging slots (row pieces of four elements), decoded once ----
    int x_pack[XS];              // word index of column 4jv | ih_l << 20 | first piece of its row << 28 | last << 29, -1 = unused
    uint32_t x_src[XS];          // byte offset from row 0 of the tile's first (image, channel)
    {
        const int x_total = P4 ? 16 * p.nti : 16 * p.nti * p.iht * (int)p.d_wv.d;
#pragma unroll
        for (int u = 0; u < XS; ++u) {
            const int e = tid + u * kBlock;
            x_pack[u] = -1; x_src[u] = 0;
            if (P4) {
                // piece = the plane of (image e / 16, channel e % 16); its window is 4 rows of 4: 8 words
                if (e < x_total && c_first + (e & 15) < g.C) {       // (channels beyond C: the window stays zero)
                    const int n_l = e >> 4, c_l = e & 15;
                    x_pack[u] = bf16_chan_off(c_l, p.ppw) + n_l * 8 + 2;
                    x_src[u] = ((n_l * g.C + c_l) * 4) * 2;
                }
            } else if (e < x_total) {
                uint32_t row, jv, c_l, rem, n_l, ih_l;
                p.d_wv.divmod(e, row, jv);
                p.d_rows.divmod(row, c_l, rem);
                p.d_iht.divmod(rem, n_l, ih_l);
                if (c_first + (int)c_l < g.C) {                      // (channels beyond C: the window stays zero)
                    x_pack[u] = (int)(bf16_chan_off(c_l, p.ppw) + ((rem * ROWP + jv * XV) >> 1)) | (int)(ih_l << 20)
                                | (jv == 0 ? 1 << 28 : 0) | (jv + 1 == p.d_wv.d ? 1 << 29 : 0);
                    x_src[u] = ((n_l * g.C + c_l) * (g.H * g.W) + jv * XV) * 2;
                }
            }
        }
    }

    uint4_t ring[GPW][MT];
    uint32_t xr[XS][XV / 2];
    uint32_t x_row_ok = 0;

    auto tile_origin = [&](int wt, bool live, const char *&dy_base, const char *&x_base, int &ih0) {
        const int w = live ? wt : wt_end - 1;
        uint32_t ng, hti;
        p.d_htiles.divmod(w, ng, hti);
        const int n0 = ng * p.nti, h0 = hti * p.ht;
        dy_base = SPARSE ? dYp + ((long)n0 * g.K + k0) * 4 : dYp + (((long)n0 * g.K + k0) * g.Ho + h0) * g.Wo * 2;
        x_base = Xp + ((long)n0 * g.C + c_first) * g.H * g.W * 2;
        ih0 = h0 - 1;
    };
    auto load_x = [&](int wt) {
        const bool live = wt < wt_end;
        const char *dyb, *xb;
        int ih0;
        tile_origin(wt, live, dyb, xb, ih0);
        x_row_ok = 0;
        if (P4) {
#pragma unroll
            for (int u = 0; u < XS; ++u) {
                const uint2 v = *(const uint2 *)(xb + (live ? x_src[u] : 0u));
                xr[u][0] = v.x; xr[u][1] = v.y;
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < XS; ++u) {
            int ih = ih0 + ((x_pack[u] >> 20) & 0xff);
            if (ih >= 0 && ih < g.H) x_row_ok |= 1u << u;
            ih = ih < 0 ? 0 : (ih >= g.H ? g.H - 1 : ih);
            const char *src = xb + (live ? x_src[u] + ih * (g.W * 2) : 0u);
            if (XV == 8) {
                const uint4_t v = *(const uint4_t *)src;
                xr[u][0] = v[0]; xr[u][1] = v[1]; xr[u][2 % (XV / 2)] = v[2]; xr[u][3 % (XV / 2)] = v[3];
            } else {
                const uint2 v = *(const uint2 *)src;
                xr[u][0] = v.x; xr[u][1] = v.y;
            }
        }
    };
    // Elements x0..x{XV-1} of piece jv belong to window columns XV*jv+1 .. XV*jv+XV (column 0 is the
    // halo): the aligned words starting at column XV*jv are (last element of the piece to the left,
    // x0), (x1, x2), ...  The left neighbour is the previous lane (pieces of a row sit in consecutive
    // lanes, and a row never straddles a group of 16 lanes); the last piece of a row also writes
    // (x{XV-1}, halo).
    // Every lane writes unconditionally (a slot without a piece, and the halo word of a piece that is not the
    // last of its row, go to a few dump words behind the tables): a conditional write masks lanes, and an
    // instruction that changes the lane mask fences the instruction scheduler, which must be free to spread
    // this work under the matrix instructions.
    uint32_t *const dump = Xs0 + 2 * p.buf_words + QT / 2;          // 8 words
    auto commit_x = [&](uint32_t *buf) {
        if (P4) {
            // rows 1 and 2 of the plane's window: (halo, x00) (x01, halo) (halo, x10) (x11, halo)
#pragma unroll
            for (int u = 0; u < XS; ++u) {
                uint32_t *w = x_pack[u] >= 0 ? buf + x_pack[u] : dump;
                w[0] = xr[u][0] << 16;
                w[1] = xr[u][0] >> 16;
                w[2] = xr[u][1] << 16;
                w[3] = xr[u][1] >> 16;
            }
            return;
        }
#pragma unroll
        for (int u = 0; u < XS; ++u) {
            const bool ok = (x_row_ok >> u) & 1;
            uint32_t r[XV / 2];
#pragma unroll
            for (int i = 0; i < XV / 2; ++i) r[i] = ok ? xr[u][i] : 0u;
            uint32_t left = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)r[XV / 2 - 1], 0x111, 0xf, 0xf, true);   // row_shr:1
            if ((x_pack[u] >> 28) & 1) left = 0u;
            uint32_t *w = x_pack[u] >= 0 ? buf + (x_pack[u] & 0xfffff) : dump;
            w[0] = __builtin_amdgcn_alignbit(r[0], left, 16);
#pragma unroll
            for (int i = 1; i < XV / 2; ++i) w[i] = __builtin_amdgcn_alignbit(r[i], r[i - 1], 16);
            uint32_t *wl = (x_pack[u] >= 0 && ((x_pack[u] >> 29) & 1)) ? w + XV / 2 : dump + XV / 2;
            *wl = r[XV / 2 - 1] >> 16;
        }
    };

    // SPARSE: sel = (position, sum) of the lane's map [and of the next image's map]; pos0 = position in
    // the map of the lane's first slot.  bf16 rounding of the sum is to nearest even.
    auto sparse_operand = [&](uint4_t sel, int pos0) -> uint4_t {
        uint4_t out{0u, 0u, 0u, 0u};
        auto put = [&](uint32_t hwv, uint32_t sbits, int first, int word0, int nslots) {
            const int rel = (int)((hwv >> 16) * g.Wo + (hwv & 0xffffu)) - first;
            const uint32_t b = (sbits + 0x7fffu + ((sbits >> 16) & 1u)) >> 16;
            const uint32_t val = (rel & 1) ? b << 16 : b;
            const bool in = (unsigned)rel < (unsigned)nslots;
#pragma unroll
            for (int w = 0; w < 4; ++w)
                if (w >= word0 && w < word0 + nslots / 2) out[w] = (in && (rel >> 1) == w - word0) ? val : 0u;
        };
        if (P4) { put(sel[0], sel[1], 0, 0, 4); put(sel[2], sel[3], 0, 2, 4); }
        else put(sel[0], sel[1], pos0, 0, 8);
        return out;
    };

    // ---- prologue: first loads, then the LDS tables and the zero fill under their latency ----
    {
        const char *dyb, *xb;
        int ih0;
        load_x(wt_begin);
        tile_origin(wt_begin, true, dyb, xb, ih0);
#pragma unroll
        for (int gi = 0; gi < GPW; ++gi)
#pragma unroll
            for (int m = 0; m < MT; ++m) ring[gi][m] = load_a(dyb + m * row_tile_bytes, a_off[gi]);
    }
    for (int q2 = tid; q2 < QT / 2; q2 += kBlock) {
        const int q = 2 * q2;
        int off = 0;
        if (q < p.q) {
            uint32_t n_l, rem, h_l, w;
            p.d_seg.divmod(q, n_l, rem);
            p.d_wo.divmod(rem, h_l, w);
            off = (n_l * p.iht * ROWP + h_l * ROWP + w) * 2;
        }
        xoffp[q2] = off;
    }
    for (int e = tid; e < (2 * p.buf_words) >> 2; e += kBlock) ((uint4_t *)Xs0)[e] = uint4_t{0u, 0u, 0u, 0u};
    const int lane_base = (c_first + i16 < g.C ? bf16_chan_off(i16, p.ppw) : 0) * 4;
    __syncthreads();
    TRACE(1);
    commit_x(Xs0);
    load_x(wt_begin + 1);
    TRACE(2);

    int par = 0;
    for (int wt = wt_begin; wt < wt_end; ++wt, par ^= 1) {
        if (wt == wt_begin + 2) TRACE(3);
        __syncthreads();   // window of tile wt is complete; everyone has left the buffer tile wt+1 goes to
        if (wt == wt_begin + 2) TRACE(4);
        if (wt == wt_begin + 3) TRACE(8);
        const char *Xw = (const char *)(Xs0 + par * p.buf_words) + lane_base;
        // The window of tile wt+1 is committed and the loads of tile wt+2 are requested after the first
        // group's operand reads, in one scheduling region with the matrix instructions of both groups (no
        // fence, no lane-mask changes inside), so that the scheduler spreads this vector and scalar work
        // under them; ahead of the matrix instructions it was a phase of its own in which the wavefront
        // issued none.
        auto stage_next = [&]() {
            commit_x(Xs0 + (par ^ 1) * p.buf_words);
            if (wt == wt_begin + 2) TRACE(5);
            load_x(wt + 2);
            if (wt == wt_begin + 2) TRACE(6);
        };
        const bool has_next = wt + 1 < wt_end;
        const char *dyb, *xb;
        int ih0;
        int flat0 = 0;                               // SPARSE: position in the map of the tile's first row
        if (SPARSE) { tile_origin(wt, true, dyb, xb, ih0); flat0 = (ih0 + 1) * g.Wo; }
        tile_origin(wt + 1, has_next, dyb, xb, ih0);

        uint32_t a_next[GPW];                       // offsets of the next tile's pieces (0: nothing to fetch)
#pragma unroll
        for (int gi = 0; gi < GPW; ++gi) a_next[gi] = has_next ? a_off[gi] : 0u;
#pragma unroll
        for (int gi = 0; gi < GPW; ++gi) {
            // pair addresses of this lane's eight positions
            const int4 po = *(const int4 *)(xoffp + first_position(gi) / 2);
            const char *a0[4] = {Xw + po.x, Xw + po.y, Xw + po.z, Xw + po.w};
            bf16x8_t a_cur[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                uint4_t v = ring[gi][m];
                if (SPARSE) v = sparse_operand(v, flat0 + a_pos[gi]);
                if (!FULL && !((a_live >> gi) & 1u)) v = uint4_t{0u, 0u, 0u, 0u};
                a_cur[m] = __builtin_bit_cast(bf16x8_t, v);
            }
            if (!FULL) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    ring[gi][m] = load_a(dyb + m * row_tile_bytes, a_next[gi]);   // same piece of the next tile
            }
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                // lo[j], hi[j]: the words of window columns (w, w+1) and (w+2, w+3) of pair j.  With
                // eight positions in one row (ROW8) the pairs are neighbours, hi[j] = lo[j+1]: the
                // five words are read as two quadruples that are the operands of taps 0 and 2 as
                // they stand; otherwise every pair has an address of its own.
                uint4_t lo, hi;
                if (ROW8) {
                    const uint32_t *wp = (const uint32_t *)(a0[0] + r * ROWP * 2);
#pragma unroll
                    for (int j = 0; j < 4; ++j) { lo[j] = wp[j]; hi[j] = wp[j + 1]; }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t *wp = (const uint32_t *)(a0[j] + r * ROWP * 2);
                        lo[j] = wp[0];
                        hi[j] = wp[1];
                    }
                }
#pragma unroll
                for (int s3 = 0; s3 < 3; ++s3) {
                    uint4_t b;
                    if (s3 == 0) b = lo;
                    else if (s3 == 2) b = hi;
                    else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) b[j] = __builtin_amdgcn_alignbit(hi[j], lo[j], 16);
                    }
                    const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, b);
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        acc[m][r * 3 + s3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_cur[m], bv, acc[m][r * 3 + s3], 0, 0, 0);
                }
            }
            if (FULL) {
                // the registers are free again: same piece of the next tile
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    ring[gi][m] = load_a(dyb + m * row_tile_bytes, a_next[gi]);
            }
            if (wt == wt_begin + 2 && gi == 0) TRACE(11);
            if (gi == 0) stage_next();
        }
        if (wt == wt_begin + 2) TRACE(7);
    }
    TRACE(9);

    // ---- epilogue, one row tile at a time: wavefronts park their accumulators in LDS (column-major,
    //      the four rows a lane holds side by side), then all threads add the four position slices
    //      and write rows of the result, coalesced ----
    {
        constexpr int KTP = 16 + 4;
        float *red = smem;                                  // [4][NCB][KTP]
        float *out = p.out[prob] + (long)split * g.K * CRS;
        const int colbase = c_first * 9;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            __syncthreads();
#pragma unroll
            for (int t = 0; t < NT; ++t)
                *(float4_t *)(red + ((wq * NCB + i16 * 9 + t) * KTP + 4 * kk)) = acc[m][t];
            __syncthreads();
            for (int o = tid; o < 4 * NCB; o += kBlock) {
                const int rq = o / NCB, lc = o % NCB;
                float4_t sum = *(const float4_t *)(red + (lc * KTP + 4 * rq));
#pragma unroll
                for (int w = 1; w < 4; ++w) sum += *(const float4_t *)(red + ((w * NCB + lc) * KTP + 4 * rq));
                const int col = colbase + lc;
                if (col < CRS) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int k = k0 + m * 16 + 4 * rq + v;
                        if (k < g.K) out[(long)k * CRS + col] = sum[v] * p.scale;
                    }
                }
            }
        }
    }
    TRACE(10);
    TRACE_BLK(1);
}

template <int GPW, int ROWP, bool FULL, bool P4, bool SPARSE>
__global__ __launch_bounds__(kBlock, 2) void wgrad_exact_bf16(const Bf16Params p)
{
    extern __shared__ float smem[];
    bf16_body<GPW, ROWP, FULL, P4, SPARSE>(p, smem, blockIdx.x, gridDim.x);
}

// A prepared launch, and a queue of them for one launch that carries several shapes.
constexpr int kBf16MultiMax = 6;        // groups per launch (their parameters are kernel arguments, 4 KB at most)
struct Bf16Launch {
    Bf16Params p;
    int gpw, rowp, full, grid;
    size_t lds;
};
struct Bf16Queue {
    SelectQueue *sel = nullptr;          // selections that must be issued before the sparse-operand launches
    int n = 0, sparse = 0;
    Bf16Launch item[kBf16MultiMax];
};

}  // namespace wgrad
