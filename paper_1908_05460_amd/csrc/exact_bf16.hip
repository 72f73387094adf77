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
    if (g.C % 16 || g.K % kBf16KT || (!p4 && (g.W % 4 || L % 8))) return false;
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
        pl.ktiles = g.K / kBf16KT; pl.ctiles = g.C / 16; pl.ctch = 16;
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

// Enqueues the kernel (not the combine); the caller has checked pointer alignment (16 bytes).
int launch_exact_bf16(const Geometry &g, const ExactPlan &pl, const Batch &b, float *const *out, hipStream_t st,
                      const SparseA *sparse)
{
    Bf16Params p{};
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
    const int grid = pl.ktiles * pl.ctiles * pl.splits * b.n;
    if (pl.gpw == 2 && pl.rowp == 4) bf16_inst<2, 4>(p, grid, pl.lds_bytes, st);
    else if (pl.gpw == 2 && pl.rowp == 12) bf16_inst<2, 12>(p, grid, pl.lds_bytes, st);
    else if (pl.gpw == 2 && pl.rowp == 20) bf16_inst<2, 20>(p, grid, pl.lds_bytes, st);
    else if (pl.gpw == 2 && pl.rowp == 36) bf16_inst<2, 36>(p, grid, pl.lds_bytes, st);
    else if (pl.gpw == 1 && pl.rowp == 8) bf16_inst<1, 8>(p, grid, pl.lds_bytes, st);
    else return WGRAD_UNSUPPORTED;
    return launch_status();
}

#if defined(WGRAD_TUNING) && !defined(WGRAD_NO_TRACE)
extern "C" int wgrad_debug_read_trace_bf16(long long *host_out)
{
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_trace), sizeof(long long) * (64 + 2 * 4096));
}
#endif

}  // namespace wgrad
