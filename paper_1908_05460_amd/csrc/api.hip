// C ABI of libwgrad (declared in include/wgrad.h): argument validation and dispatch.
// Everything here runs on the host; validation precedes the first launch.
#include <mutex>

#include "exact_stream_kernel.hpp"

using namespace wgrad;

static int make_geometry(const wgrad_conv_desc *d, Geometry &g)
{
    if (!d) return WGRAD_INVALID_ARG;
    if (d->N <= 0 || d->C <= 0 || d->H <= 0 || d->W <= 0 || d->K <= 0 || d->R <= 0 || d->S <= 0)
        return WGRAD_INVALID_ARG;
    if (d->stride_h <= 0 || d->stride_w <= 0 || d->pad_h < 0 || d->pad_w < 0) return WGRAD_INVALID_ARG;
    if (d->dtype != WGRAD_F32 && d->dtype != WGRAD_BF16) return WGRAD_INVALID_ARG;
    // output extent in 64-bit before anything is narrowed: a huge padding must not wrap
    const long ho = ((long)d->H + 2 * (long)d->pad_h - d->R) / d->stride_h + 1;
    const long wo = ((long)d->W + 2 * (long)d->pad_w - d->S) / d->stride_w + 1;
    if ((long)d->H + 2 * (long)d->pad_h < d->R || (long)d->W + 2 * (long)d->pad_w < d->S) return WGRAD_INVALID_ARG;  // empty output
    // (row, col) of a map is packed in 32 bits; window arithmetic of the kernels is 32-bit
    if (ho < 1 || wo < 1 || ho >= 32768 || wo >= 32768) return WGRAD_UNSUPPORTED;
    if (d->pad_h >= 32768 || d->pad_w >= 32768 || d->stride_h >= 32768 || d->stride_w >= 32768 ||
        d->R >= 32768 || d->S >= 32768) return WGRAD_UNSUPPORTED;
    g.N = d->N; g.C = d->C; g.H = d->H; g.W = d->W; g.K = d->K; g.R = d->R; g.S = d->S;
    g.sh = d->stride_h; g.sw = d->stride_w; g.ph = d->pad_h; g.pw = d->pad_w;
    g.Ho = (int)ho;
    g.Wo = (int)wo;
    g.bf16 = d->dtype == WGRAD_BF16;
    // index arithmetic inside the kernels is 32-bit per tensor dimension product below
    const long lim = 1l << 31;
    if ((long)g.N * g.K >= lim || (long)g.Ho * g.Wo >= lim || g.dw_elems() >= lim || (long)g.H * g.W >= lim)
        return WGRAD_UNSUPPORTED;
    return WGRAD_OK;
}

static bool ws_ok(const void *ws, size_t have, size_t need)
{
    if (need == 0) return true;
    return ws != nullptr && have >= need && ((uintptr_t)ws % kAlign) == 0;
}

extern "C" {

int conv_wgrad_exact(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                     void *ws, size_t ws_bytes, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!X || !dY || !dW) return WGRAD_INVALID_ARG;
    const ExactPlan pl = plan_exact(g);
    if (!pl.ok) return WGRAD_UNSUPPORTED;
    if (!ws_ok(ws, ws_bytes, pl.ws_bytes)) return WGRAD_WORKSPACE_TOO_SMALL;
    Batch b{};
    b.n = 1; b.X[0] = X; b.dY[0] = dY; b.dW[0] = dW;
    return launch_exact(g, pl, b, ws, (hipStream_t)stream);
}

int conv_wgrad_approx(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                      float scale, int32_t *idx_out, float *sum_out,
                      void *ws, size_t ws_bytes, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!X || !dY || !dW) return WGRAD_INVALID_ARG;
    const ApproxPlan pl = plan_approx(g);
    if (!ws_ok(ws, ws_bytes, pl.ws_bytes)) return WGRAD_WORKSPACE_TOO_SMALL;
    Batch b{};
    b.n = 1; b.X[0] = X; b.dY[0] = dY; b.dW[0] = dW;
    return launch_approx(g, pl, b, scale, idx_out, sum_out, ws, (hipStream_t)stream);
}

int conv_wgrad_approx_topk(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                           int topk, float scale, int32_t *idx_out, float *sum_out,
                           void *ws, size_t ws_bytes, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!X || !dY || !dW) return WGRAD_INVALID_ARG;
    if (!topk_supported(g, topk)) return WGRAD_UNSUPPORTED;
    if (!ws_ok(ws, ws_bytes, topk_ws_bytes(g, topk))) return WGRAD_WORKSPACE_TOO_SMALL;
    return launch_approx_topk(g, X, dY, dW, topk, scale, idx_out, sum_out, ws, (hipStream_t)stream);
}

size_t conv_wgrad_topk_workspace_bytes(const wgrad_conv_desc *desc, int topk)
{
    Geometry g;
    if (make_geometry(desc, g) != WGRAD_OK || !topk_supported(g, topk)) return 0;
    return topk_ws_bytes(g, topk);
}

int conv_wgrad_approx_nhwc(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                           wgrad_dw_layout dw_layout, float scale, int32_t *idx_out, float *sum_out,
                           void *ws, size_t ws_bytes, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!X || !dY || !dW || !dw_layout_ok(dw_layout)) return WGRAD_INVALID_ARG;
    if (!ws_ok(ws, ws_bytes, approx_nhwc_ws_bytes(g))) return WGRAD_WORKSPACE_TOO_SMALL;
    return launch_approx_nhwc(g, X, dY, dW, dw_layout, scale, idx_out, sum_out, ws, (hipStream_t)stream);
}

int conv_wgrad_exact_nhwc(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                          wgrad_dw_layout dw_layout, void *ws, size_t ws_bytes, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!X || !dY || !dW || !dw_layout_ok(dw_layout)) return WGRAD_INVALID_ARG;
    const ExactPlan pl = plan_exact(g);
    if (!pl.ok) return WGRAD_UNSUPPORTED;
    if (!ws_ok(ws, ws_bytes, exact_nhwc_ws_bytes(g, pl))) return WGRAD_WORKSPACE_TOO_SMALL;
    return launch_exact_nhwc(g, pl, X, dY, dW, dw_layout, ws, (hipStream_t)stream);
}

size_t conv_wgrad_nhwc_workspace_bytes(const wgrad_conv_desc *desc, wgrad_method method)
{
    Geometry g;
    if (make_geometry(desc, g) != WGRAD_OK) return 0;
    if (method == WGRAD_EXACT) { const ExactPlan pl = plan_exact(g); return pl.ok ? exact_nhwc_ws_bytes(g, pl) : 0; }
    if (method == WGRAD_APPROX) return approx_nhwc_ws_bytes(g);
    return 0;
}

int conv_wgrad_transpose_x(const wgrad_conv_desc *desc, int to_nhwc, const void *src, void *dst, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!src || !dst || src == dst) return WGRAD_INVALID_ARG;
    return launch_transpose_x(g, to_nhwc != 0, src, dst, (hipStream_t)stream);
}

int conv_wgrad_permute_dw(const wgrad_conv_desc *desc, wgrad_dw_layout from, wgrad_dw_layout to,
                          const float *src, float *dst, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!src || !dst || src == dst || !dw_layout_ok(from) || !dw_layout_ok(to)) return WGRAD_INVALID_ARG;
    return launch_permute_dw(g, from, to, src, dst, (hipStream_t)stream);
}

int conv_wgrad_select(const wgrad_conv_desc *desc, const void *dY, int32_t *idx, float *sum, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!dY || !idx || !sum) return WGRAD_INVALID_ARG;
    return launch_select(g, dY, idx, sum, (hipStream_t)stream);
}

int conv_wgrad_zero(const wgrad_conv_desc *desc, float *dW, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!dW) return WGRAD_INVALID_ARG;
    return launch_zero(dW, g.dw_elems(), (hipStream_t)stream);
}

int conv_wgrad_random(const wgrad_conv_desc *desc, float *dW, float sigma, uint64_t seed,
                      uint64_t offset, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!dW || !(sigma >= 0.0f)) return WGRAD_INVALID_ARG;
    return launch_random(dW, g.dw_elems(), sigma, seed, offset, (hipStream_t)stream);
}

size_t conv_wgrad_workspace_bytes(const wgrad_conv_desc *desc, wgrad_method method)
{
    Geometry g;
    if (make_geometry(desc, g) != WGRAD_OK) return 0;
    if (method == WGRAD_EXACT) { const ExactPlan pl = plan_exact(g); return pl.ok ? pl.ws_bytes : 0; }
    if (method == WGRAD_APPROX) return plan_approx(g).ws_bytes;
    return 0;
}

}  // extern "C"

// ---- schedule: layers with the same geometry and method are folded into one launch ----
namespace {

bool same_desc(const wgrad_conv_desc &a, const wgrad_conv_desc &b)
{
    return a.N == b.N && a.C == b.C && a.H == b.H && a.W == b.W && a.K == b.K && a.R == b.R && a.S == b.S &&
           a.stride_h == b.stride_h && a.stride_w == b.stride_w && a.pad_h == b.pad_h && a.pad_w == b.pad_w &&
           a.dtype == b.dtype;
}

// group[i] = index of the first layer of i's group; a group holds at most kMaxBatch exact or
// approx layers of identical descriptor (zero and random layers are never grouped)
void make_groups(const wgrad_conv_desc *layers, const uint8_t *method, int n, int *group)
{
    for (int i = 0; i < n; ++i) group[i] = -1;
    for (int i = 0; i < n; ++i) {
        if (group[i] >= 0) continue;
        group[i] = i;
        if (method[i] != WGRAD_EXACT && method[i] != WGRAD_APPROX) continue;
        int members = 1;
        for (int j = i + 1; j < n && members < kMaxBatch; ++j)
            if (group[j] < 0 && method[j] == method[i] && same_desc(layers[i], layers[j])) { group[j] = i; ++members; }
    }
}

size_t method_ws(const Geometry &g, int method)
{
    if (method == WGRAD_EXACT) { const ExactPlan pl = plan_exact(g); return pl.ok ? pl.ws_bytes : 0; }
    if (method == WGRAD_APPROX) return plan_approx(g).ws_bytes;
    return 0;
}

}  // namespace

// topk > 0: approximated layers take the top-k form, one launch sequence each (they are not folded into groups);
// a layer whose maps have fewer than topk positions keeps all of them
static int layer_topk(const Geometry &g, int topk)
{
    const long L = (long)g.Ho * g.Wo;
    return (long)topk < L ? topk : (int)L;
}

// Approximated layers of one shape stay a group only where the fused top-k kernel takes the shape (it is the one
// top-k form that runs several layers in one launch); the workspace is a slice per layer either way.
static void make_groups_topk(const wgrad_conv_desc *layers, const uint8_t *method, int n, int topk, int *group)
{
    make_groups(layers, method, n, group);
    if (topk <= 0) return;
    for (int i = 0; i < n; ++i) {
        if (method[i] != WGRAD_APPROX || group[i] != i) continue;
        Geometry g;
        if (make_geometry(&layers[i], g) == WGRAD_OK && topk_takes_fused(g, layer_topk(g, topk))) continue;
        for (int j = i + 1; j < n; ++j)
            if (group[j] == i) group[j] = j;
    }
}

static size_t schedule_ws_bytes(const wgrad_conv_desc *layers, const uint8_t *method, int32_t nlayers, int topk)
{
    if (!layers || !method || nlayers <= 0 || nlayers > 4096) return 0;
    int group[4096];
    make_groups_topk(layers, method, nlayers, topk, group);
    size_t need = 0;
    for (int i = 0; i < nlayers; ++i) {
        if (group[i] != i) continue;
        Geometry g;
        if (make_geometry(&layers[i], g) != WGRAD_OK) return 0;
        int members = 0;
        for (int j = i; j < nlayers; ++j) members += group[j] == i;
        if (topk > 0 && method[i] == WGRAD_APPROX) {
            need += align_up(topk_ws_bytes(g, layer_topk(g, topk))) * members;
            continue;
        }
        need += align_up(method_ws(g, method[i])) * members;       // every group keeps its partials until the final reduction
    }
    return need;
}

extern "C" size_t conv_wgrad_schedule_workspace_bytes(const wgrad_conv_desc *layers, const uint8_t *method, int32_t nlayers)
{
    return schedule_ws_bytes(layers, method, nlayers, 0);
}

extern "C" size_t conv_wgrad_schedule_topk_workspace_bytes(const wgrad_conv_desc *layers, const uint8_t *method,
                                                           int32_t nlayers, int32_t topk)
{
    return topk >= 1 && topk <= kTopKMax ? schedule_ws_bytes(layers, method, nlayers, topk) : 0;
}

static int schedule_run_impl(const wgrad_conv_desc *layers, const void *const *X, const void *const *dY,
                             float *const *dW, const uint8_t *method, int32_t nlayers, int topk, float scale,
                             float sigma, uint64_t seed, uint64_t offset, void *ws, size_t ws_bytes,
                             void *stream)
{
    if (!layers || !X || !dY || !dW || !method || nlayers <= 0 || nlayers > 4096) return WGRAD_INVALID_ARG;
    // pass 1: validate every layer before anything is enqueued
    for (int i = 0; i < nlayers; ++i) {
        Geometry g;
        int rc = make_geometry(&layers[i], g);
        if (rc != WGRAD_OK) return rc;
        if (method[i] > WGRAD_RANDOM) return WGRAD_INVALID_ARG;
        if (!dW[i]) return WGRAD_INVALID_ARG;
        if (method[i] == WGRAD_EXACT || method[i] == WGRAD_APPROX) {
            if (!X[i] || !dY[i]) return WGRAD_INVALID_ARG;
            if (method[i] == WGRAD_EXACT && !plan_exact(g).ok) return WGRAD_UNSUPPORTED;
        } else if (method[i] == WGRAD_RANDOM && !(sigma >= 0.0f)) {
            return WGRAD_INVALID_ARG;
        }
    }
    if (!ws_ok(ws, ws_bytes, schedule_ws_bytes(layers, method, nlayers, topk))) return WGRAD_WORKSPACE_TOO_SMALL;

    // pass 2: enqueue on the caller's stream: one launch sequence per group of exact or approximated
    // layers, then one reduction of all their partial results, then the zero and the random fills
    hipStream_t st = (hipStream_t)stream;
    int group[4096];
    make_groups_topk(layers, method, nlayers, topk, group);
    CombineQueue queue;
    MultiQueue multi;
    int nexact = 0;
    for (int i = 0; i < nlayers; ++i) nexact += method[i] == WGRAD_EXACT && group[i] == i;
    MultiQueue *mq = nexact > 1 && tune_int("WGRAD_MULTI", 1) ? &multi : nullptr;
    // workgroups of a multi-shape launch are shared out to the groups in proportion to their work
    double exact_flops = 0;
    auto group_flops = [&](int i) {
        double f = 0;
        for (int j = i; j < nlayers; ++j)
            if (group[j] == i) {
                Geometry gj;
                make_geometry(&layers[j], gj);
                double w = 2.0 * gj.N * gj.K * gj.Ho * gj.Wo * (double)gj.crs();
                // layers that are not bound by the matrix core take longer than their FLOPs say: a handful of
                // input channels (bound by the dY stream), strides (a window four times the tile)
                if (gj.C < 16) w *= tune_int("WGRAD_MULTI_W_FLAT", 20) / 10.0;
                if (gj.sh > 1 || gj.sw > 1) w *= tune_int("WGRAD_MULTI_W_STRIDE", 25) / 10.0;
                // 4x4 planes: their tiles are half as long (the window of eight images does not fit next to a
                // second workgroup's), so a FLOP takes longer there even with the halo-only taps left out (swept)
                const int wc = plan_exact(gj).wc;
                if (wc == 1) w *= tune_int("WGRAD_MULTI_W_WC1", 125) / 100.0;
                if (wc == 2) w *= tune_int("WGRAD_MULTI_W_WC2", 100) / 100.0;
                f += w;
            }
        return f;
    };
    if (mq)
        for (int i = 0; i < nlayers; ++i)
            if (method[i] == WGRAD_EXACT && group[i] == i) {
                Geometry gi;
                make_geometry(&layers[i], gi);
                if (!plan_exact(gi).plane2) exact_flops += group_flops(i);   // (those groups have a launch of their own)
            }
    int napprox = 0;
    for (int i = 0; i < nlayers; ++i) napprox += topk == 0 && method[i] == WGRAD_APPROX && group[i] == i;
    int ntopk = 0;
    for (int i = 0; i < nlayers; ++i) ntopk += topk > 0 && method[i] == WGRAD_APPROX;
    FusedQueue *fq = (napprox > 1 || ntopk > 1) && tune_int("WGRAD_FUSED_MULTI", 1) ? fused_queue_new() : nullptr;
    SelectQueue *sq = napprox > 1 && tune_int("WGRAD_SELECT_MULTI", 1) ? select_queue_new() : nullptr;
    GatherQueue *gq = napprox > 1 && tune_int("WGRAD_GATHER_MULTI", 1) ? gather_queue_new(sq) : nullptr;
    // groups that run on the bf16 matrix core (exact ones, and approximated ones through the sparse operand)
    // are collected for launches that carry several shapes
    // (a group alone keeps its own launch: it has to fill the chip by itself)
    int nbf16 = 0;
    for (int i = 0; i < nlayers; ++i) {
        if ((method[i] != WGRAD_EXACT && method[i] != WGRAD_APPROX) || group[i] != i || layers[i].dtype != WGRAD_BF16) continue;
        Geometry g;
        make_geometry(&layers[i], g);
        nbf16 += method[i] == WGRAD_EXACT ? plan_exact(g).mm16 : (topk == 0 ? plan_approx(g).mm : 0);
    }
    Bf16Queue *bq = nbf16 > 1 && tune_int("WGRAD_BF16_MULTI", 1) ? bf16_queue_new(sq) : nullptr;
    char *ws_next = (char *)ws;
    int rc = WGRAD_OK;
    for (int i = 0; i < nlayers && rc == WGRAD_OK; ++i) {
        if ((method[i] != WGRAD_EXACT && method[i] != WGRAD_APPROX) || group[i] != i) continue;
        Geometry g;
        make_geometry(&layers[i], g);
        Batch b{};
        for (int j = i; j < nlayers; ++j)
            if (group[j] == i) { b.X[b.n] = X[j]; b.dY[b.n] = dY[j]; b.dW[b.n] = dW[j]; ++b.n; }
        if (method[i] == WGRAD_EXACT) {
            int share = 0;
            // 768 in all -- three per CU, all resident at once, so a workgroup's fixed cost is paid once per CU
            // slot -- while a workgroup's share stays near 100 us; stacks with more work than that get two or
            // three rounds of 768, which evens out the groups' different speeds at the end of the launch
            // (VGG-19 at N = 128, 102 GFLOP: 768 -> 2304 workgroups, exact phase -7 %)
            if (mq) {
                int rounds = (int)(exact_flops / 34e9 + 0.5);
                rounds = rounds < 1 ? 1 : (rounds > 3 ? 3 : rounds);
                share = (int)(tune_int("WGRAD_MULTI_TOTAL", 768 * rounds) * group_flops(i) / exact_flops + 0.5);
            }
            rc = launch_exact(g, plan_exact(g), b, ws_next, st, &queue, mq, share < 8 ? 8 : share, bq);
        }
        else if (topk > 0) {
            const int k = layer_topk(g, topk);
            const size_t slice = align_up(topk_ws_bytes(g, k));
            // a group of layers in one fused launch where that form takes them; otherwise layer by layer
            if (!(b.n > 1 && launch_topk_group(g, b, k, scale, ws_next, slice, st, &rc, fq, &queue)))
                for (int j = 0; j < b.n && rc == WGRAD_OK; ++j)
                    rc = launch_approx_topk(g, b.X[j], b.dY[j], b.dW[j], k, scale, nullptr, nullptr,
                                            ws_next + (size_t)j * slice, st, fq, &queue);
            ws_next += slice * b.n;
            continue;
        }
        else rc = launch_approx(g, plan_approx(g), b, scale, nullptr, nullptr, ws_next, st, &queue, fq, bq, gq, sq);
        ws_next += align_up(method_ws(g, method[i])) * b.n;
    }
    if (sq) {
        if (rc == WGRAD_OK) rc = select_flush(*sq, st);
    }
    if (rc == WGRAD_OK && mq) rc = multi_flush(multi, st);
    if (bq) {
        if (rc == WGRAD_OK) rc = bf16_flush(*bq, st);
        bf16_queue_delete(bq);
    }
    if (gq) {
        if (rc == WGRAD_OK) rc = gather_flush(*gq, st);
        gather_queue_delete(gq);
    }
    if (sq) select_queue_delete(sq);
    if (fq) {
        if (rc == WGRAD_OK) rc = fused_flush(*fq, st);
        fused_queue_delete(fq);
    }
    if (rc == WGRAD_OK) rc = combine_flush(queue, st);
    // fills, kTableMax tensors per launch
    for (int which = WGRAD_ZERO; which <= WGRAD_RANDOM && rc == WGRAD_OK; ++which) {
        float *dst[kTableMax];
        long elems[kTableMax];
        uint64_t offs[kTableMax];
        int n = 0;
        uint64_t off = offset;
        for (int i = 0; i <= nlayers && rc == WGRAD_OK; ++i) {
            if (n == kTableMax || (i == nlayers && n > 0)) {
                rc = which == WGRAD_ZERO ? launch_zero_table(dst, elems, n, st)
                                         : launch_random_table(dst, elems, offs, n, sigma, seed, st);
                n = 0;
            }
            if (i == nlayers) break;
            const long e = (long)layers[i].K * layers[i].C * layers[i].R * layers[i].S;
            if (method[i] == which) { dst[n] = dW[i]; elems[n] = e; offs[n] = off; ++n; }
            off += (uint64_t)e;
        }
    }
    return rc;
}

extern "C" int conv_wgrad_schedule_run(const wgrad_conv_desc *layers, const void *const *X, const void *const *dY,
                            float *const *dW, const uint8_t *method, int32_t nlayers, float scale,
                            float sigma, uint64_t seed, uint64_t offset, void *ws, size_t ws_bytes,
                            void *stream)
{
    return schedule_run_impl(layers, X, dY, dW, method, nlayers, 0, scale, sigma, seed, offset, ws, ws_bytes, stream);
}

extern "C" int conv_wgrad_schedule_run_topk(const wgrad_conv_desc *layers, const void *const *X, const void *const *dY,
                                 float *const *dW, const uint8_t *method, int32_t nlayers, int32_t topk, float scale,
                                 float sigma, uint64_t seed, uint64_t offset, void *ws, size_t ws_bytes,
                                 void *stream)
{
    if (topk < 1 || topk > kTopKMax) return WGRAD_UNSUPPORTED;
    return schedule_run_impl(layers, X, dY, dW, method, nlayers, topk, scale, sigma, seed, offset, ws, ws_bytes, stream);
}

// ---- the approximation for callers that cannot allocate ----
// The scratch memory of conv_wgrad_approx_static lives in the library's own device image: every GPU the library
// runs on holds its copy of this array, at its own address, until the process ends.  `scratch` is only a
// host-side stand-in for the symbol; the memory is reached through the per-device address looked up below.
static __device__ __align__(256) unsigned char scratch[WGRAD_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];           // device address of `scratch` on device i, once looked up

// The array's address on the current device (looked up on the first call per device), or nullptr.
void *static_scratch_of_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

extern "C" int conv_wgrad_approx_static(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                                        float scale, int32_t *idx_out, float *sum_out, void *stream)
{
    Geometry g;
    int rc = make_geometry(desc, g);
    if (rc != WGRAD_OK) return rc;
    if (!X || !dY || !dW) return WGRAD_INVALID_ARG;
    const ApproxPlan pl = plan_approx(g);
    if (pl.ws_bytes > (size_t)WGRAD_STATIC_SCRATCH_BYTES) return WGRAD_SCRATCH_LIMIT;
    // nothing in the approximation's kernels reads scratch it has not written in the same call (positions, sums
    // and every partial result are overwritten), so the array's old contents need no clearing
    void *ws = pl.ws_bytes ? static_scratch_of_current_device() : nullptr;
    if (pl.ws_bytes && !ws) return WGRAD_LAUNCH_FAILED;
    Batch b{};
    b.n = 1; b.X[0] = X; b.dY[0] = dY; b.dW[0] = dW;
    return launch_approx(g, pl, b, scale, idx_out, sum_out, ws, (hipStream_t)stream);
}

extern "C" {

const char *conv_wgrad_status_string(int status)
{
    switch (status) {
        case WGRAD_OK: return "ok";
        case WGRAD_INVALID_ARG: return "invalid argument (null pointer, non-positive size, empty output, bad dtype or method)";
        case WGRAD_UNSUPPORTED: return "unsupported: a size beyond the kernels' 32-bit index ranges, or top-k out of range";
        case WGRAD_WORKSPACE_TOO_SMALL: return "workspace too small or not 256-byte aligned";
        case WGRAD_LAUNCH_FAILED: return "the HIP runtime refused a kernel launch";
        case WGRAD_SCRATCH_LIMIT: return "the layer needs more scratch memory than the library's static buffer (WGRAD_STATIC_SCRATCH_BYTES) holds";
        default: return "unknown status";
    }
}

}  // extern "C"
