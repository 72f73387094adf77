// Host side of the bf16 matrix-core exact-gradient kernel: tile plan and launch.
#define WGRAD_TRACE_HERE
#include "exact_bf16_kernel.hpp"

namespace wgrad {

static int largest_divisor_upto(int n, int limit)
{
    if (limit >= n) return n;
    for (int d = limit; d >= 1; --d)
        if (n % d == 0) return d;
    return 1;
}

// (GPW, ROWP) pairs that are instantiated
static bool bf16_has_inst(int gpw, int rowp)
{
    return gpw == 2 ? (rowp == 4 || rowp == 12 || rowp == 20 || rowp == 36) : (gpw == 1 && rowp == 8);
}

// Fills the plan for the bf16 matrix-core form; false if the shape is outside what it handles
// (the fp32 matrix-core kernels then take it).
bool plan_exact_bf16(const Geometry &g, ExactPlan &pl)
{
    if (!g.bf16 || g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1) return false;
    const int L = g.Ho * g.Wo;
    const bool p4 = g.H == 2 && g.W == 2;               // 2x2 planes have a staging path of their own
    // (any number of input channels: a last tile of fewer than 16 multiplies zeros for the rest -- still a third of the
    //  fp32 matrix core's time on the three channels of a first layer)
    if ((g.C % 16 && !tune_int("WGRAD_BF16_ANY_C", 1)) || g.K % kBf16KT || (!p4 && (g.W % 4 || L % 8))) return false;
    const int iwt = g.Wo + 2;
    const int rowp = p4 ? 4 : (iwt <= 8 ? 8 : (iwt <= 12 ? 12 : (iwt <= 20 ? 20 : (iwt <= 36 ? 36 : 0))));
    if (!rowp) return false;
    for (int gpw = 2; gpw >= 1; --gpw) {
        if (!bf16_has_inst(gpw, rowp)) continue;
        const int qt = 128 * gpw;
        int nti, ht;
        if (L >= qt) { nti = 1; ht = largest_divisor_upto(g.Ho, qt / g.Wo < 1 ? 1 : qt / g.Wo); }
        else { ht = g.Ho; nti = largest_divisor_upto(g.N, qt / L < 1 ? 1 : qt / L); }
        const int q = nti * ht * g.Wo;
        if (q > qt || (!p4 && (ht * g.Wo) % 8 != 0) || (p4 && nti % 2 != 0)) continue;
        const int iht = ht + 2;
        int ppw = (nti * iht * rowp + 1) / 2;
        while (ppw % 32 != 1) ++ppw;
        const int buf_words = 4 * (4 * ppw + 12);
        size_t lds = ((size_t)2 * buf_words + qt / 2 + 8) * 4;      // two windows, the pair-offset table, 8 dump words
        const size_t red = (size_t)4 * 144 * 20 * 4;               // epilogue exchange buffer [4][144][20]
        if (red > lds) lds = red;
        const int xv = p4 ? 4 : bf16_xv(rowp);
        if (!p4 && g.W % xv != 0) continue;
        const long x_slots = p4 ? (long)16 * nti : (long)16 * nti * iht * (g.W / xv);
        if (lds > 80 * 1024 || x_slots > (long)bf16_xslots(gpw, rowp) * kBlock || iht > 255) continue;   // two workgroups per CU
        if ((long)nti * g.K * L * 2 >= (1l << 31) || (long)nti * g.C * g.H * g.W * 2 >= (1l << 31)) continue;
        pl.mm16 = 1; pl.stream = 0; pl.gpw = gpw; pl.xv = xv;
        pl.nt = 9; pl.wk = 1; pl.tap_mode = 1;
        pl.ktiles = g.K / kBf16KT; pl.ctiles = (g.C + 15) / 16; pl.ctch = 16;
        pl.nti = nti; pl.ht = ht; pl.q = q; pl.qpad = qt; pl.qp = 0;
        pl.iht = iht; pl.iwt = iwt; pl.pp = ppw; pl.xbuf = buf_words; pl.rowp = rowp;
        pl.lds_bytes = lds;
        return true;
    }
    return false;
}

template <int GPW, int ROWP, bool FULL, bool SPARSE>
static void bf16_inst2(const Bf16Params &p, int grid, size_t lds, hipStream_t st)
{
    constexpr bool P4 = ROWP == 4;
    // more than 64 KB of dynamic LDS has to be granted per kernel function (the CU has 160 KB)
    if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)wgrad_exact_bf16<GPW, ROWP, FULL, P4, SPARSE>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return;
    WGRAD_LAUNCH((wgrad_exact_bf16<GPW, ROWP, FULL, P4, SPARSE>), dim3(grid), dim3(kBlock), lds, st, p);
}

template <int GPW, int ROWP>
static void bf16_inst(const Bf16Params &p, int grid, size_t lds, hipStream_t st)
{
    const bool sparse = p.hw[0] != nullptr;
    if (p.q == 128 * GPW) {
        if (sparse) bf16_inst2<GPW, ROWP, true, true>(p, grid, lds, st);
        else bf16_inst2<GPW, ROWP, true, false>(p, grid, lds, st);
    } else {
        if (sparse) bf16_inst2<GPW, ROWP, false, true>(p, grid, lds, st);
        else bf16_inst2<GPW, ROWP, false, false>(p, grid, lds, st);
    }
}

static int bf16_launch_now(const Bf16Launch &L, hipStream_t st)
{
    if (L.gpw == 2 && L.rowp == 4) bf16_inst<2, 4>(L.p, L.grid, L.lds, st);
    else if (L.gpw == 2 && L.rowp == 12) bf16_inst<2, 12>(L.p, L.grid, L.lds, st);
    else if (L.gpw == 2 && L.rowp == 20) bf16_inst<2, 20>(L.p, L.grid, L.lds, st);
    else if (L.gpw == 2 && L.rowp == 36) bf16_inst<2, 36>(L.p, L.grid, L.lds, st);
    else if (L.gpw == 1 && L.rowp == 8) bf16_inst<1, 8>(L.p, L.grid, L.lds, st);
    else return WGRAD_UNSUPPORTED;
    return launch_status();
}

// ---- one launch for several shapes: the groups of a run each fill the chip once (512 workgroups, all resident), so
//      back to back every group pays its ramp and its tail with most of the chip idle; as one grid, the workgroups of
//      the next group start as those of the current one finish.  A workgroup looks its group up in the kernel arguments
//      (read through the kernel-argument segment pointer: indexing the by-value argument with a run-time group number
//      would make the compiler copy all of it to scratch memory) and runs that group's instantiation of the body. ----
struct Bf16Multi {
    int n;
    int begin[kBf16MultiMax + 1];    // first workgroup of each group (multiples of 8: the XCD numbering of a group
                                     // then starts on XCD 0); begin[n] = grid size
    int count[kBf16MultiMax];        // workgroups of the group
    int variant[kBf16MultiMax];
    Bf16Params p[kBf16MultiMax];
};
static_assert(sizeof(Bf16Multi) <= 4096, "kernel arguments");

// (id, GPW, ROWP, FULL)
#define WGRAD_BF16_VARIANTS(X) \
    X(0, 2, 4, false) X(1, 2, 4, true) X(2, 2, 12, false) X(3, 2, 12, true) X(4, 2, 20, false) X(5, 2, 20, true) \
    X(6, 2, 36, false) X(7, 2, 36, true) X(8, 1, 8, false) X(9, 1, 8, true)

static int bf16_variant(int gpw, int rowp, int full)
{
#define X(ID, GPW, ROWP, FULL) if (gpw == GPW && rowp == ROWP && (full != 0) == FULL) return ID;
    WGRAD_BF16_VARIANTS(X)
#undef X
    return -1;
}

template <bool SPARSE>
__global__ __launch_bounds__(kBlock, 2) void wgrad_exact_bf16_multi(const Bf16Multi)
{
    extern __shared__ float smem[];
    const Bf16Multi *mp = (const Bf16Multi *)__builtin_amdgcn_kernarg_segment_ptr();
    const int n = mp->n;
    int gi = 0;
    for (int i = 1; i < n; ++i) gi += (int)blockIdx.x >= mp->begin[i];
    const int bid = (int)blockIdx.x - mp->begin[gi], nblk = mp->count[gi];
    if (bid >= nblk) return;
    const Bf16Params &p = mp->p[gi];
    switch (mp->variant[gi]) {
#define X(ID, GPW, ROWP, FULL) case ID: bf16_body<GPW, ROWP, FULL, ROWP == 4, SPARSE>(p, smem, bid, nblk); break;
        WGRAD_BF16_VARIANTS(X)
#undef X
        default: break;
    }
}

Bf16Queue *bf16_queue_new(SelectQueue *selects)
{
    Bf16Queue *q = new Bf16Queue();
    q->sel = selects;
    return q;
}
void bf16_queue_delete(Bf16Queue *q) { delete q; }

int bf16_flush(Bf16Queue &q, hipStream_t st)
{
    if (q.n == 0) return WGRAD_OK;
    if (q.sel) {
        const int rc = select_flush(*q.sel, st);
        if (rc != WGRAD_OK) return rc;
    }
    if (q.n == 1) {
        q.n = 0;
        return bf16_launch_now(q.item[0], st);
    }
    Bf16Multi m{};
    m.n = q.n;
    size_t lds = 0;
    int blocks = 0;
    for (int i = 0; i < q.n; ++i) {
        const Bf16Launch &L = q.item[i];
        m.begin[i] = blocks;
        m.count[i] = L.grid;
        m.variant[i] = bf16_variant(L.gpw, L.rowp, L.full);
        m.p[i] = L.p;
        blocks += (L.grid + 7) / 8 * 8;
        if (L.lds > lds) lds = L.lds;
    }
    m.begin[q.n] = blocks;
    const bool sparse = q.sparse;
    q.n = 0;
    if (sparse) {
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)wgrad_exact_bf16_multi<true>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return WGRAD_LAUNCH_FAILED;
        WGRAD_LAUNCH((wgrad_exact_bf16_multi<true>), dim3((unsigned)blocks), dim3(kBlock), lds, st, m);
    } else {
        if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)wgrad_exact_bf16_multi<false>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return WGRAD_LAUNCH_FAILED;
        WGRAD_LAUNCH((wgrad_exact_bf16_multi<false>), dim3((unsigned)blocks), dim3(kBlock), lds, st, m);
    }
    return launch_status();
}

// Enqueues the kernel (not the combine); the caller has checked pointer alignment (16 bytes).  With a queue the
// launch is only recorded there (bf16_flush issues it, together with the others recorded).
int launch_exact_bf16(const Geometry &g, const ExactPlan &pl, const Batch &b, float *const *out, hipStream_t st,
                      const SparseA *sparse, Bf16Queue *queue)
{
    Bf16Launch L{};
    Bf16Params &p = L.p;
    for (int i = 0; i < kMaxBatch; ++i) {          // unused slots repeat problem 0
        const int j = i < b.n ? i : 0;
        p.X[i] = b.X[j]; p.dY[i] = b.dY[j]; p.out[i] = out[j];
        p.hw[i] = sparse ? sparse->hw[j] : nullptr;
        p.sum[i] = sparse ? sparse->sum[j] : nullptr;
    }
    p.scale = sparse ? sparse->scale : 1.0f;
    p.per_prob = pl.ktiles * pl.ctiles * pl.splits;
    p.g = g;
    p.ktiles = pl.ktiles; p.ctiles = pl.ctiles; p.splits = pl.splits;
    p.nti = pl.nti; p.ht = pl.ht; p.q = pl.q; p.iht = pl.iht;
    p.h_tiles = pl.h_tiles; p.n_groups = pl.n_groups;
    p.seg = pl.ht * g.Wo;
    p.ppw = pl.pp; p.buf_words = pl.xbuf; p.rowp = pl.rowp;
    p.d_wv = FastDiv(g.W >= pl.xv ? g.W / pl.xv : 1);
    p.d_rows = FastDiv(pl.nti * pl.iht);
    p.d_iht = FastDiv(pl.iht);
    p.d_seg = FastDiv(p.seg);
    p.d_wo = FastDiv(g.Wo);
    p.d_htiles = FastDiv(pl.h_tiles);
    L.gpw = pl.gpw; L.rowp = pl.rowp; L.full = pl.q == 128 * pl.gpw;
    L.grid = pl.ktiles * pl.ctiles * pl.splits * b.n;
    L.lds = pl.lds_bytes;
    if (bf16_variant(L.gpw, L.rowp, L.full) < 0) return WGRAD_UNSUPPORTED;
    if (!queue) return bf16_launch_now(L, st);
    if (queue->n == kBf16MultiMax || (queue->n > 0 && queue->sparse != (sparse != nullptr))) {
        const int rc = bf16_flush(*queue, st);
        if (rc != WGRAD_OK) return rc;
    }
    queue->sparse = sparse != nullptr;
    queue->item[queue->n++] = L;
    return WGRAD_OK;
}


}  // namespace wgrad

WGRAD_TRACE_READER(wgrad_debug_read_trace_bf16)
