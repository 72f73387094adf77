// Shared host/device declarations of libwgrad (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <vector>

#include "wgrad.h"
#ifdef WGRAD_TUNING
#include "dev_tuning.hpp"
#endif

namespace wgrad {

constexpr int kBlock = 256;          // threads per workgroup: 4 wavefronts of 64
constexpr int kWave = 64;
constexpr int kNumXCD = 8;           // MI355X: 8 accelerator dies, each with its own L2
constexpr int kNumCU = 256;
constexpr size_t kAlign = 256;       // workspace carve-out alignment
constexpr int kMaxBatch = 8;         // layers of identical shape a schedule run folds into one launch

// Tensors of up to kMaxBatch problems of identical geometry handled by one launch.
struct Batch {
    int n;
    const void *X[kMaxBatch];
    const void *dY[kMaxBatch];
    float *dW[kMaxBatch];
};

// Division of a small unsigned number by a run-time constant: q = umulhi(n, m)
// with m = floor(2^32/d) + 1 is exact while n*d < 2^32 (the host checks that
// bound for every divisor it builds).
struct FastDiv {
    uint32_t d, m, one;              // one = all ones when d == 1 (then m = 0), else 0: keeps div() branch-free
    __host__ __device__ FastDiv() : d(1), m(0), one(0xffffffffu) {}
    __host__ explicit FastDiv(uint32_t div)
        : d(div), m(div > 1 ? (uint32_t)((1ull << 32) / div) + 1u : 0u), one(div > 1 ? 0u : 0xffffffffu) {}
    __device__ __forceinline__ uint32_t div(uint32_t n) const { return __umulhi(n, m) | (n & one); }
    __device__ __forceinline__ void divmod(uint32_t n, uint32_t &q, uint32_t &r) const {
        q = div(n);
        r = n - q * d;
    }
};

struct Geometry {                    // validated convolution geometry
    int N, C, H, W, K, R, S, sh, sw, ph, pw, Ho, Wo;
    int bf16;                        // element type of X and dY
    __host__ __device__ long crs() const { return (long)C * R * S; }
    __host__ __device__ long dw_elems() const { return (long)K * C * R * S; }
};

// Tuning constants are written tune_int("NAME", value): in this build that is the value.  (Development builds
// define WGRAD_TUNING and take the definitions below from dev_tuning.hpp instead, which lets an environment
// variable override a constant and adds timestamp traces.)
#ifndef WGRAD_TUNING
constexpr int tune_int(const char *, int dflt) { return dflt; }
#define TRACE(i) do { } while (0)
#define TRACE_BLK(which) do { } while (0)
#define FTRACE(i) do { } while (0)
#define FTRACE_G(gi) do { } while (0)
#define FTRACE_SET(i, v) do { (void)(v); } while (0)
#define FTRACE_CLOCK() 0ll
#define WGRAD_TRACE_READER(name)
#define WGRAD_FUSED_TRACE_READER(name)
#endif

inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }

// Physical workgroup id -> logical id such that the workgroups resident on one
// XCD (ids congruent modulo 8 are dispatched to the same die) own a contiguous
// range of logical ids, so neighbours in the logical order share that die's L2.
__device__ __forceinline__ int xcd_contiguous_id(int bid, int nblocks)
{
    const int q = nblocks / kNumXCD, rem = nblocks % kNumXCD;
    const int xcd = bid % kNumXCD, local = bid / kNumXCD;
    return xcd * q + (xcd < rem ? xcd : rem) + local;
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// ---- internal launchers (host). Each validates nothing: the C ABI layer did. ----
struct ExactPlan {
    int nt, wk, tap_mode;            // MFMA column tiles per wave, waves along K, column mapping
    int ktiles, ctiles, splits;
    int nti, ht, q, qpad, qp;        // images / output rows / positions per staged tile, LDS pitch of dY rows
    int iht, iwt, pp, ctch;          // staged input rows / cols, LDS pitch of an X channel, channels staged
    int h_tiles, n_groups;
    int xv;                          // elements per staging access (4, 2; 0 = element-wise staging)
    int stream, gpw, xbuf, rowp;           // streaming form: A operand from global memory, window double-buffered
    int wc;                          // streaming form: column-uniform position order with this many 4-column blocks per output row (0: row-major order)
    int img4;                        // streaming form, 4x4 planes: image-uniform position order (a step contracts one position of four images)
    int mm16;                        // bf16 matrix-core form of the streaming kernel
    int direct;                      // general form: no tile of whole output rows fits the LDS
    int plane2;                      // 2x2 planes, fp32: the plain matrix product over (position, element) pairs
    size_t lds_bytes, ws_bytes;
    bool ok;
};
ExactPlan plan_exact(const Geometry &g, bool allow_stream = true);
bool plan_exact_stream(const Geometry &g, ExactPlan &pl);
struct MultiQueue;
int launch_exact_stream(const Geometry &g, const ExactPlan &pl, const Batch &b, float *const *out, hipStream_t st,
                        MultiQueue *mq = nullptr);
bool plan_exact_bf16(const Geometry &g, ExactPlan &pl);
bool plane2_takes(const Geometry &g);
struct MultiQueue;
int launch_exact_plane2(const Geometry &g, const Batch &b, hipStream_t st, MultiQueue *mq = nullptr);
struct CombineQueue;
void plan_exact_direct(const Geometry &g, ExactPlan &pl);
int launch_exact_direct(const Geometry &g, const ExactPlan &pl, const void *X, const void *dY, float *dW, void *ws,
                        hipStream_t st, CombineQueue *defer);
// The A operand of the bf16 matrix-core kernel given as the sparsified gradient of the
// approximation: per problem, every map's selected position (row << 16 | col) and sum.
struct SparseA {
    const int32_t *hw[kMaxBatch];
    const float *sum[kMaxBatch];
    float scale;                     // applied by the kernel when it writes dW itself (one split)
};
// launches of the bf16 matrix-core kernel collected for one launch that carries several shapes
struct Bf16Queue;
struct SelectQueue;
Bf16Queue *bf16_queue_new(SelectQueue *selects = nullptr);
void bf16_queue_delete(Bf16Queue *q);
int bf16_flush(Bf16Queue &q, hipStream_t st);
int launch_exact_bf16(const Geometry &g, const ExactPlan &pl, const Batch &b, float *const *out, hipStream_t st,
                      const SparseA *sparse = nullptr, Bf16Queue *queue = nullptr);
// bf16 inputs on 2x2 and 4x4 planes: the position-major matrix-core kernel (no split, writes dW itself)
bool planes_bf16_takes(const Geometry &g);
int launch_exact_bf16_planes(const Geometry &g, const Batch &b, hipStream_t st, const SparseA *sparse = nullptr);
struct CombineQueue;
int launch_exact(const Geometry &g, const ExactPlan &pl, const Batch &b, void *ws, hipStream_t st,
                 CombineQueue *defer = nullptr, MultiQueue *mq = nullptr, int mq_blocks = 0, Bf16Queue *bq = nullptr);
int choose_splits(const ExactPlan &pl, int nprob, int want_blocks = 0);
size_t exact_ws_per_problem(const Geometry &g, const ExactPlan &pl);

struct ApproxPlan {
    int chunks, chunk_n;             // batch chunks whose partial sums are combined afterwards
    int use_lds, fused, m, nb, pitch, wp, ctiles, ktiles;   // LDS form of the gather: tile shape
    int mm;                          // contraction on the bf16 matrix core from the selection results
    int sx;                          // fp32, planes of up to four positions: exact kernel on the sparsified dY
    ExactPlan ex;                    // its plan
    size_t off_idx, off_sum, off_part, off_sparse, ws_bytes;
};
ApproxPlan plan_approx(const Geometry &g, bool allow_lds = true, bool allow_fused = true, bool allow_mm = true);
struct FusedQueue;
struct GatherQueue;
// selections of several layer groups collected for one launch; the queues of their consumers (the LDS gathers, the
// sparse-operand launches of the bf16 matrix-core kernel) issue it before they issue themselves
struct SelectQueue;
SelectQueue *select_queue_new();
void select_queue_delete(SelectQueue *q);
int select_flush(SelectQueue &q, hipStream_t st);
int launch_select(const Geometry &g, const void *dY, int32_t *idx, float *sum, hipStream_t st);
int launch_approx(const Geometry &g, const ApproxPlan &pl, const Batch &b, float scale,
                  int32_t *idx_out, float *sum_out, void *ws, hipStream_t st, CombineQueue *defer = nullptr,
                  FusedQueue *fq = nullptr, Bf16Queue *bq = nullptr, GatherQueue *gq = nullptr,
                  SelectQueue *sq = nullptr);
// LDS-form gathers of several layer groups, collected for one launch
GatherQueue *gather_queue_new(SelectQueue *selects = nullptr);
void gather_queue_delete(GatherQueue *q);
int gather_flush(GatherQueue &q, hipStream_t st);
// groups of layers that the fused approximation kernel takes, collected for one launch
FusedQueue *fused_queue_new();
void fused_queue_delete(FusedQueue *q);
int fused_flush(FusedQueue &q, hipStream_t st);

// top-k form of the approximation (k kept positions per map, each carrying sum/k)
constexpr int kTopKMax = 64;
bool topk_supported(const Geometry &g, int k);
size_t topk_ws_bytes(const Geometry &g, int k);
size_t topk_borrowed_partial_bytes(const Geometry &g);
bool topk_takes_fused(const Geometry &g, int k);
bool topk_fused(const Geometry &g, const Batch &b, int k, float scale,
                int32_t *idx_out, float *sum_out, float *partials, long partial_stride, hipStream_t st, int *rc,
                FusedQueue *fq = nullptr, CombineQueue *defer = nullptr);
// layers of one geometry of a schedule run through the fused top-k form in one group; false if the form does not
// take them (the caller then runs them one by one).  ws: the members' workspace slices, slice_bytes apart.
bool launch_topk_group(const Geometry &g, const Batch &b, int k, float scale, void *ws, size_t slice_bytes,
                       hipStream_t st, int *rc, FusedQueue *fq, CombineQueue *defer);
bool topk_gather_lds(const Geometry &g, const void *X, const int32_t *hw, const float *sum, int k, float scale,
                     float *dW, float *partials, size_t partial_cap_bytes, hipStream_t st, int *rc);
int launch_approx_topk(const Geometry &g, const void *X, const void *dY, float *dW, int k, float scale,
                       int32_t *idx_out, float *sum_out, void *ws, hipStream_t st, FusedQueue *fq = nullptr,
                       CombineQueue *defer = nullptr);

// channel-last input and the other filter-gradient layouts (Section 2.4)
bool dw_layout_ok(int layout);
size_t approx_nhwc_ws_bytes(const Geometry &g);
int launch_approx_nhwc(const Geometry &g, const void *X, const void *dY, float *dW, int dw_layout, float scale,
                       int32_t *idx_out, float *sum_out, void *ws, hipStream_t st);
size_t exact_nhwc_ws_bytes(const Geometry &g, const ExactPlan &pl);
int launch_exact_nhwc(const Geometry &g, const ExactPlan &pl, const void *X, const void *dY, float *dW,
                      int dw_layout, void *ws, hipStream_t st);
int launch_transpose_x(const Geometry &g, bool to_nhwc, const void *src, void *dst, hipStream_t st);
int launch_permute_dw(const Geometry &g, int from, int to, const float *src, float *dst, hipStream_t st);

// Reductions of partial results that a run of several layers postpones: every producer writes
// its partials into a workspace region of its own, and one table-driven launch at the end
// reduces all of them (a launch per layer group costs more than the reduction itself).
constexpr int kTableMax = 32;        // tensors one table-driven launch handles
struct CombineItem {
    const float *part;               // [nparts][elems]
    float *dW;
    int nparts, elems;
    float scale;
};
struct CombineQueue {              // grows as needed; nothing is launched before combine_flush
    std::vector<CombineItem> item;
};
int combine_flush(CombineQueue &q, hipStream_t st);

// dW[i][o] = scale * sum_j partials[i * prob_stride + j * elems + o] for the nprob problems of a batch;
// with a queue the work is only recorded there
int launch_combine(const float *partials, long prob_stride, int nparts, long elems, float scale,
                   float *const *dW, int nprob, hipStream_t st, CombineQueue *defer = nullptr);
int launch_zero(float *dW, long elems, hipStream_t st);
int launch_random(float *dW, long elems, float sigma, uint64_t seed, uint64_t offset, hipStream_t st);
// the same for up to kTableMax tensors in one launch (offset[i]: first counter of tensor i)
int launch_zero_table(float *const *dW, const long *elems, int n, hipStream_t st);
int launch_random_table(float *const *dW, const long *elems, const uint64_t *offset, int n, float sigma,
                        uint64_t seed, hipStream_t st);

// hipGetLastError() reports the last error of ANY earlier runtime call on this thread, so it
// is cleared before a launch and read right after it.
inline void clear_launch_error() { (void)hipGetLastError(); }
inline int launch_status() { return hipGetLastError() == hipSuccess ? WGRAD_OK : WGRAD_LAUNCH_FAILED; }
#define WGRAD_LAUNCH(...)                                                                   \
    do {                                                                                    \
        ::wgrad::clear_launch_error();                                                      \
        hipLaunchKernelGGL(__VA_ARGS__);                                                    \
    } while (0)

}  // namespace wgrad
