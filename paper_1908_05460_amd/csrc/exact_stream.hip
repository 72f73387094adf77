// Host side of the streaming exact-gradient kernel: tile plan and launch.
#include "exact_stream_kernel.hpp"

namespace wgrad {

// ------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------
static int stream_pitch(int len)   // smallest pitch >= len with pitch % 32 == 1
{
    int p = len;
    while (p % 32 != 1) ++p;
    return p;
}

static int largest_divisor_le(int n, int limit)
{
    if (limit >= n) return n;
    for (int d = limit; d >= 1; --d)
        if (n % d == 0) return d;
    return 1;
}

// Fills the streaming-form fields of the plan; returns false if the shape is outside what the
// streaming kernel handles (the staged kernel then takes it).
bool plan_exact_stream(const Geometry &g, ExactPlan &pl)
{
    const int WQ = 4 / pl.wk;
    const int L = g.Ho * g.Wo;
    const int xv = g.W % 4 == 0 ? 4 : (g.W % 2 == 0 ? 2 : 0);
    if (!xv || L % 4 != 0) return false;
    for (int gpw = 8; gpw >= 2; gpw /= 2) {
        const int qt = 16 * gpw * WQ;
        int nti, ht;
        if (L >= qt) { nti = 1; ht = largest_divisor_le(g.Ho, qt / g.Wo < 1 ? 1 : qt / g.Wo); }
        else { ht = g.Ho; nti = largest_divisor_le(g.N, qt / L < 1 ? 1 : qt / L); }
        const int q = nti * ht * g.Wo;
        if (q > qt || (ht * g.Wo) % 4 != 0) continue;
        if (q * 2 <= qt && gpw == 8) continue;             // more than half the tile would be padding: try the smaller one
        const int iht = (ht - 1) * g.sh + g.R, iwt = (g.Wo - 1) * g.sw + g.S;
        // 3x3 tap mode: a fixed row pitch (4 mod 8, so that rows too spread over the banks) makes the
        // tap offsets compile-time constants; otherwise rows are packed
        int rowp = iwt;
        if (pl.tap_mode && pl.nt == 9) {
            const int fixed = iwt <= 4 ? 4 : (iwt <= 12 ? 12 : (iwt <= 20 ? 20 : (iwt <= 36 ? 36 : 0)));
            if (fixed && stream_has_rowp(fixed, xv)) rowp = fixed;
        }
        // 4x4 planes, tiles of eight whole images: image-uniform order.  The lane groups of an operand read then address
        // different images and the same row, so the rows are packed (pitch 6: the window of eight images fits next to
        // two other workgroups' only so) and the images' windows are placed 4 (mod 8) floats apart, which spreads the
        // 64 lanes over all banks
        const bool img4 = tune_int("WGRAD_STREAM_IMG4", 1) && !g.bf16 && pl.tap_mode && pl.nt == 9 && pl.wk == 4 && xv == 4
                          && gpw == 8 && g.R == 3 && g.S == 3 && g.sh == 1 && g.sw == 1 && g.ph == 1 && g.pw == 1
                          && g.Ho == 4 && g.Wo == 4 && nti == 8 && ht == 4;
        if (img4) rowp = 6;
        int ipitch = iht * rowp;
        if (img4) while (ipitch % 8 != 4) ++ipitch;
        const int pp = stream_pitch(nti * ipitch);
        const int xbuf = (pl.ctch + 3) / 4 * (4 * pp + 4);        // quads of channels, see stream_chan_off
        size_t lds = ((size_t)2 * xbuf + qt) * 4;
        const size_t red = (size_t)WQ * (pl.nt * 16) * (16 * pl.wk + 4) * 4;    // epilogue exchange buffer [WQ][NT*16][KT + 4]
        if (red > lds) lds = red;
        const long x_slots = (long)pl.ctch * nti * iht * (g.W / xv);
        // up to 64 KB two workgroups share a CU; a larger window (strided layers) gets a CU to itself
        const size_t lds_cap = (size_t)tune_int("WGRAD_STREAM_LDS_KB", 64) * 1024;
        if (lds > lds_cap || x_slots > (long)stream_xslots(pl.wk, gpw) * kBlock || iht > 255 || (long)xbuf >= (1 << 20)) continue;
        if ((long)nti * g.K * L * 4 >= (1l << 31) || (long)nti * g.C * g.H * g.W * 4 >= (1l << 31)) continue;
        pl.stream = 1; pl.gpw = gpw; pl.xv = xv;
        pl.img4 = img4;
        // column-uniform position order (the taps that meet only the zero halo are left out): 3x3, stride 1,
        // padding 1, rows of four or eight positions, K tiles of 64, whole blocks of four rows
        pl.wc = 0;
        if (tune_int("WGRAD_STREAM_WC", 1) && !g.bf16 && pl.tap_mode && pl.nt == 9 && xv == 4
            && (pl.wk == 4 || (pl.wk == 2 && g.Wo == 16 && tune_int("WGRAD_STREAM_WC_K32", 1)))
            && g.R == 3 && g.S == 3 && g.sh == 1 && g.sw == 1 && g.ph == 1 && g.pw == 1
            && ((g.Wo == 4 && gpw == 4 && rowp == 12) || img4 || (g.Wo == 8 && gpw == 8 && rowp == 12)
                || (tune_int("WGRAD_STREAM_WC_WIDE", 1) && ((g.Wo == 16 && gpw == 8 && rowp == 20) || (g.Wo == 32 && gpw == 8 && rowp == 36))))
            && ht % 4 == 0 && q % 16 == 0)
            pl.wc = g.Wo / 4;
        pl.nti = nti; pl.ht = ht; pl.q = q; pl.qpad = qt; pl.qp = 0;
        pl.iht = iht; pl.iwt = iwt; pl.pp = pp; pl.xbuf = xbuf; pl.rowp = rowp;
        pl.lds_bytes = lds;
        return true;
    }
    return false;
}

int launch_stream_now(const StreamLaunch &L, hipStream_t st)
{
    if (L.plane2) launch_plane2_kernel(L, st);
    else if (L.wk == 1) stream_launch_w1(L.p, L.nt, L.xv, L.gpw, L.rowp_inst, L.grid, L.lds, st);
    else if (L.wk == 2) stream_launch_w2(L.p, L.nt, L.xv, L.gpw, L.rowp_inst, L.grid, L.lds, st);
    else stream_launch_w4(L.p, L.nt, L.xv, L.gpw, L.rowp_inst, L.grid, L.lds, st);
    return launch_status();
}

// Enqueues the streaming kernel (not the combine); the caller has checked pointer alignment.  With a
// queue, fp32 launches of a shape that a multi-shape launch can carry are only recorded there.
int launch_exact_stream(const Geometry &g, const ExactPlan &pl, const Batch &b, float *const *out, hipStream_t st,
                        MultiQueue *mq)
{
    StreamLaunch L{};
    StreamShape &p = L.p.s;
    for (int i = 0; i < kMaxBatch; ++i) {          // unused slots repeat problem 0
        const int j = i < b.n ? i : 0;
        L.p.X[i] = b.X[j]; L.p.dY[i] = b.dY[j]; L.p.out[i] = out[j];
    }
    L.nprob = b.n;
    p.per_prob = pl.ktiles * pl.ctiles * pl.splits;
    p.g = g;
    p.tap_mode = pl.tap_mode; p.ktiles = pl.ktiles; p.ctiles = pl.ctiles; p.splits = pl.splits;
    p.nti = pl.nti; p.ht = pl.ht; p.q = pl.q; p.iht = pl.iht; p.iwt = pl.iwt; p.pp = pl.pp; p.ctch = pl.ctch;
    p.h_tiles = pl.h_tiles; p.n_groups = pl.n_groups;
    p.seg = pl.ht * g.Wo;
    p.xbuf = pl.xbuf;
    p.rowp = pl.rowp;
    p.wc = pl.wc;
    p.img4 = pl.img4;
    p.ipitch = pl.iht * pl.rowp;
    if (pl.img4) while (p.ipitch % 8 != 4) ++p.ipitch;
    p.d_gpi = FastDiv(pl.wc ? (pl.ht / 4) * pl.wc : 1);
    p.d_wv = FastDiv(g.W / pl.xv);
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
            p.tile_toff[t] = (tap / g.S) * pl.rowp + tap % g.S;
            p.tile_tap[t] = tap;
        }
    L.grid = pl.ktiles * pl.ctiles * pl.splits * b.n;
    L.rowp_inst = stream_has_rowp(pl.rowp, pl.xv) && pl.nt == 9 && pl.tap_mode ? pl.rowp : 0;
    L.nt = pl.nt; L.wk = pl.wk; L.xv = pl.xv; L.gpw = pl.gpw; L.lds = pl.lds_bytes;
    L.wc = L.rowp_inst ? pl.wc : 0;
    L.img4 = L.wc == 1 ? pl.img4 : 0;
    p.wc = L.wc;
    // up to three workgroups per CU must fit next to each other for a mixed launch to pay
    if (mq && !g.bf16 && L.lds <= 52 * 1024 && multi_variant(L.nt, L.wk, L.xv, L.gpw, L.rowp_inst, L.wc, L.img4) >= 0) {
        if (mq->n >= tune_int("WGRAD_MULTI_GROUPS", kMultiMax) || mq->tensors + b.n > kMultiTensors) {
            const int rc = multi_flush(*mq, st);
            if (rc != WGRAD_OK) return rc;
        }
        mq->item[mq->n++] = L;
        mq->tensors += b.n;
        return WGRAD_OK;
    }
    return launch_stream_now(L, st);
}

}  // namespace wgrad
