// Max Gradient Approximation (Algorithm 1 of arXiv 1908.05460) on gfx950.
//
//   select :  for every map dY[n,k,:,:]   idx = argmax |dY| (lowest flat position on
//             ties),  S = signed sum of the map                  -- streams dY once
//   gather :  dW[k,c,r,s] = scale * sum_n S[n,k] * X[n,c,h* sh + r - ph, w* sw + s - pw]
//             (zero outside X)                                    -- reads the patches
//   combine:  sums the batch-chunk partials of the gather (shared with the exact path).
#include <algorithm>

#define WGRAD_TRACE_FUSED_HERE
#include "common.hpp"

namespace wgrad {

// ------------------------------------------------------------------------------------
// select: a group of G lanes (power of two, <= 64) owns one map; each lane walks the
// map in 16-byte pieces G pieces apart, keeps its own best (|v| bits, position) and
// partial sum, then the group reduces with a butterfly over lane-xor shuffles.
//
// The comparison is done on the magnitude bits as unsigned integers, which orders
// finite floats (and infinities) exactly as |v| does; +0/-0 and +v/-v compare equal.
// A NaN gets key 0: it ranks as a zero of the map (lowest position among equal keys wins).
// Ties go to the lowest position: within a lane positions are visited in ascending
// order with a strict '>', and across lanes the packed key (mag << 32 | ~pos) is
// maximised, which prefers the larger magnitude and then the smaller position.
// ------------------------------------------------------------------------------------
template <bool BF16>
__device__ __forceinline__ uint32_t mag_key(uint32_t bits)   // bits of the value as fp32
{
    const uint32_t m = bits & 0x7fffffffu;
    return m > 0x7f800000u ? 0u : m;
}

// Reductions over the 64 lanes of a wavefront with data-parallel-primitive moves (no LDS, a few cycles per step):
// an inclusive scan inside each row of 16 lanes (shifts by 1, 2, 4, 8), then lane 15 of row 0 is folded into row 1 and
// of row 2 into row 3 (row_bcast:15), then lane 31 into rows 2 and 3 (row_bcast:31); lane 63 holds the result, which is
// returned as a wavefront-uniform value.  Lanes without a source keep the identity (0 for both operations used here).
// All 64 lanes must be active.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = max(v, dpp_move<0x111, 0xf>(v));     // row_shr:1
    v = max(v, dpp_move<0x112, 0xf>(v));     // row_shr:2
    v = max(v, dpp_move<0x114, 0xf>(v));     // row_shr:4
    v = max(v, dpp_move<0x118, 0xf>(v));     // row_shr:8
    v = max(v, dpp_move<0x142, 0xa>(v));     // row_bcast:15 into rows 1 and 3
    v = max(v, dpp_move<0x143, 0xc>(v));     // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
__device__ __forceinline__ float wave_sum_f32(float v)
{
    v += __uint_as_float(dpp_move<0x111, 0xf>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x112, 0xf>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x114, 0xf>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x118, 0xf>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x142, 0xa>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x143, 0xc>(__float_as_uint(v)));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// The largest (magnitude key, inverted position) pair of the wavefront, lexicographically: first the largest key, then,
// among the lanes that hold it, the largest inverted position (the smallest position).  A lane without a candidate
// passes (0, 0); a real inverted position is never 0.
// The same scans stopped after the row steps: lane 15 of each row of 16 lanes ends with its row's result.
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v)
{
    v = max(v, dpp_move<0x111, 0xf>(v));
    v = max(v, dpp_move<0x112, 0xf>(v));
    v = max(v, dpp_move<0x114, 0xf>(v));
    v = max(v, dpp_move<0x118, 0xf>(v));
    return v;
}
__device__ __forceinline__ float row_sum_f32(float v)
{
    v += __uint_as_float(dpp_move<0x111, 0xf>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x112, 0xf>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x114, 0xf>(__float_as_uint(v)));
    v += __uint_as_float(dpp_move<0x118, 0xf>(__float_as_uint(v)));
    return v;
}

__device__ __forceinline__ void wave_max_pair(uint32_t key, uint32_t inv_pos, uint32_t &key_max, uint32_t &inv_pos_max)
{
    key_max = wave_max_u32(key);
    inv_pos_max = wave_max_u32(key == key_max ? inv_pos : 0u);
}

// Per-problem pointers of a batched approximation launch (problem = blockIdx.y or .z).
struct ApproxBatch {
    const void *X[kMaxBatch];
    const void *dY[kMaxBatch];
    int32_t *hw[kMaxBatch];      // packed (row << 16 | col) of every map
    float *sum[kMaxBatch];       // signed sum of every map
    float *out[kMaxBatch];       // dW, or the batch-chunk partials
};

// (bx, by): the workgroup's number within its problem, and the problem
template <bool BF16, int VEC>
__device__ __forceinline__ void select_body(const ApproxBatch &ab, long maps, int len, int Wo, int G,
                                            int32_t *__restrict__ flat_out, float *__restrict__ sum_b, int bx, int by)
{
    // flat_out / sum_b: optional user outputs, single-problem launches only
    const void *__restrict__ dY = ab.dY[by];
    int32_t *__restrict__ hw_out = ab.hw[by];
    float *__restrict__ sum_a = ab.sum[by];
    const int lane = threadIdx.x & 63;
    const int maps_per_wave = 64 / G;
    const long wave_global = (long)bx * (kBlock / 64) + (threadIdx.x >> 6);
    const long map = wave_global * maps_per_wave + lane / G;
    const int gl = lane % G;

    uint32_t best_key = 0, best_pos = 0;
    bool have = false;
    float sum = 0.f;
    if (map < maps) {
        const long base = map * len;
#pragma unroll 4
        for (int e = gl * VEC; e < len; e += G * VEC) {
            uint32_t bits[VEC];
            if (VEC == 1) {
                bits[0] = BF16 ? (uint32_t)((const uint16_t *)dY)[base + e] << 16
                               : ((const uint32_t *)dY)[base + e];
            } else if (BF16) {   // VEC == 8 : one 16-byte load of 8 bf16
                const uint4 raw = *(const uint4 *)((const uint16_t *)dY + base + e);
                const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) { bits[2 * i] = w[i] << 16; bits[2 * i + 1] = w[i] & 0xffff0000u; }
            } else {             // VEC == 4 : one 16-byte load of 4 fp32
                const uint4 raw = *(const uint4 *)((const uint32_t *)dY + base + e);
                bits[0] = raw.x; bits[1] = raw.y; bits[2] = raw.z; bits[3] = raw.w;
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                const uint32_t key = mag_key<BF16>(bits[i]);
                if (!have || key > best_key) { best_key = key; best_pos = e + i; have = true; }
                sum += __uint_as_float(bits[i]);
            }
        }
    }
    // lanes that saw nothing (len smaller than the group's reach) must lose every comparison
    unsigned long long packed = have ? ((unsigned long long)best_key << 32) | (uint32_t)~best_pos : 0ull;
    for (int d = G >> 1; d > 0; d >>= 1) {
        const unsigned long long other = __shfl_xor(packed, d, 64);
        const float osum = __shfl_xor(sum, d, 64);
        packed = other > packed ? other : packed;
        sum += osum;
    }
    if (map < maps && gl == 0) {
        const int32_t pos = (int32_t)~(uint32_t)packed;
        if (flat_out) flat_out[map] = pos;
        if (hw_out) hw_out[map] = ((pos / Wo) << 16) | (pos % Wo);   // (row, col), for the gather
        if (sum_a) sum_a[map] = sum;
        if (sum_b) sum_b[map] = sum;
    }
}

template <bool BF16, int VEC>
__global__ __launch_bounds__(kBlock) void approx_select(ApproxBatch ab, long maps, int len,
                                                        int Wo, int G, int32_t *__restrict__ flat_out,
                                                        float *__restrict__ sum_b)
{
    select_body<BF16, VEC>(ab, maps, len, Wo, G, flat_out, sum_b, blockIdx.x, blockIdx.y);
}

// The selections of several layer groups of a schedule run as one grid (each is a few microseconds of HBM
// streaming; launched one by one they are mostly ramp and tail).  Group table in the kernel arguments, read in place.
constexpr int kSelectMultiMax = 6;
struct SelectGroup {
    ApproxBatch ab;
    long maps;
    int len, Wo, G, gx;              // gx: workgroups per problem
};
struct SelectMulti {
    int n;
    int begin[kSelectMultiMax + 1];  // first workgroup of each group; begin[n] = grid size
    SelectGroup grp[kSelectMultiMax];
};

template <bool BF16, int VEC>
__global__ __launch_bounds__(kBlock) void approx_select_multi(const SelectMulti)
{
    const SelectMulti *mp = (const SelectMulti *)__builtin_amdgcn_kernarg_segment_ptr();
    const int n = mp->n;
    int gi = 0;
    for (int i = 1; i < n; ++i) gi += (int)blockIdx.x >= mp->begin[i];
    const SelectGroup &G = mp->grp[gi];
    const int linear = (int)blockIdx.x - mp->begin[gi];
    select_body<BF16, VEC>(G.ab, G.maps, G.len, G.Wo, G.G, nullptr, nullptr, linear % G.gx, linear / G.gx);
}

struct SelectQueue {
    int n = 0, bf16 = 0, vec = 0;
    int nprob[kSelectMultiMax];
    SelectGroup grp[kSelectMultiMax];
};

SelectQueue *select_queue_new() { return new SelectQueue; }
void select_queue_delete(SelectQueue *q) { delete q; }

int select_flush(SelectQueue &q, hipStream_t st)
{
    if (q.n == 0) return WGRAD_OK;
    SelectMulti m{};
    m.n = q.n;
    long blocks = 0;
    for (int i = 0; i < q.n; ++i) {
        m.grp[i] = q.grp[i];
        m.begin[i] = (int)blocks;
        blocks += (long)q.grp[i].gx * q.nprob[i];
    }
    m.begin[q.n] = (int)blocks;
    const int bf16 = q.bf16, vec = q.vec;
    q.n = 0;
    if (blocks >= (1l << 31)) return WGRAD_UNSUPPORTED;
#define SM_ARGS dim3((unsigned)blocks), dim3(kBlock), 0, st, m
    if (bf16) { if (vec == 8) WGRAD_LAUNCH((approx_select_multi<true, 8>), SM_ARGS); else WGRAD_LAUNCH((approx_select_multi<true, 1>), SM_ARGS); }
    else      { if (vec == 4) WGRAD_LAUNCH((approx_select_multi<false, 4>), SM_ARGS); else WGRAD_LAUNCH((approx_select_multi<false, 1>), SM_ARGS); }
#undef SM_ARGS
    return launch_status();
}

// With a queue (and no user outputs) the launch is only recorded there; select_flush issues it with the others.
static int launch_select_impl(const Geometry &g, const ApproxBatch &ab, int nprob, int32_t *flat_out,
                              float *sum_b, hipStream_t st, SelectQueue *sq = nullptr)
{
    const int len = g.Ho * g.Wo;
    const long maps = (long)g.N * g.K;
    const int full = g.bf16 ? 8 : 4;                      // elements per 16-byte access
    bool vec_ok = len % full == 0;
    for (int i = 0; i < nprob; ++i) vec_ok = vec_ok && ((uintptr_t)ab.dY[i] % 16) == 0;
    const int vec = vec_ok ? full : 1;
    // lanes per map: enough that each lane issues about four accesses
    int G = 1;
    while (G < 64 && G * vec * 4 < len) G <<= 1;
    const long waves = (maps + 64 / G - 1) / (64 / G);
    const int grid = (int)((waves + kBlock / 64 - 1) / (kBlock / 64));
    if (sq && !flat_out && !sum_b) {
        if (sq->n == kSelectMultiMax || (sq->n > 0 && (sq->bf16 != g.bf16 || sq->vec != vec))) {
            const int rc = select_flush(*sq, st);
            if (rc != WGRAD_OK) return rc;
        }
        SelectGroup &S = sq->grp[sq->n];
        sq->nprob[sq->n++] = nprob;
        sq->bf16 = g.bf16; sq->vec = vec;
        S.ab = ab; S.maps = maps; S.len = len; S.Wo = g.Wo; S.G = G; S.gx = grid;
        return WGRAD_OK;
    }
#define SEL_ARGS dim3(grid, nprob), dim3(kBlock), 0, st, ab, maps, len, g.Wo, G, flat_out, sum_b
    if (g.bf16) {
        if (vec == 8) WGRAD_LAUNCH((approx_select<true, 8>), SEL_ARGS);
        else          WGRAD_LAUNCH((approx_select<true, 1>), SEL_ARGS);
    } else {
        if (vec == 4) WGRAD_LAUNCH((approx_select<false, 4>), SEL_ARGS);
        else          WGRAD_LAUNCH((approx_select<false, 1>), SEL_ARGS);
    }
#undef SEL_ARGS
    return launch_status();
}

int launch_select(const Geometry &g, const void *dY, int32_t *idx, float *sum, hipStream_t st)
{
    ApproxBatch ab{};
    ab.dY[0] = dY; ab.sum[0] = sum;           // no packed positions wanted
    return launch_select_impl(g, ab, 1, idx, nullptr, st);
}

// Maps of up to four positions (2x2 planes), fp32: one thread per map selects, sums and writes the map's
// sparsified form -- the scaled sum at the selected position, zeros elsewhere.  The approximated gradient is the
// exact gradient of that tensor (Section 2.4), and on planes this small the matrix-core kernel computes it faster
// than a gather does (a quarter of the positions survive; the gather moves as much data as the exact kernel).
__global__ __launch_bounds__(kBlock) void sparsify_small(ApproxBatch ab, long maps, int len, float scale,
                                                         int32_t *__restrict__ flat_out, float *__restrict__ sum_b)
{
    const long map = (long)blockIdx.x * kBlock + threadIdx.x;
    if (map >= maps) return;
    const uint32_t *__restrict__ dY = (const uint32_t *)ab.dY[blockIdx.y] + map * len;
    float *__restrict__ sparse = ab.out[blockIdx.y] + map * len;
    uint32_t best_key = 0;
    int best_pos = 0;
    float sum = 0.f;
    for (int e = 0; e < len; ++e) {
        const uint32_t bits = dY[e];
        const uint32_t key = mag_key<false>(bits);
        if (key > best_key) { best_key = key; best_pos = e; }
        sum += __uint_as_float(bits);
    }
    for (int e = 0; e < len; ++e) sparse[e] = e == best_pos ? sum * scale : 0.f;
    if (flat_out) flat_out[map] = best_pos;
    if (sum_b) sum_b[map] = sum;
}

// ------------------------------------------------------------------------------------
// gather, direct form: one thread per filter-gradient entry (k, c, r, s) and batch
// chunk; it walks the chunk's images, reads the map's (row, col, S) and the one input
// element its tap sees.  Used when the patches touch only part of each input plane
// (few output channels, large planes) and for filters other than 3x3.
// ------------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(kBlock) void approx_gather_direct(ApproxBatch ab, Geometry g,
                                                               int chunk_n, float scale)
{
    const void *__restrict__ X = ab.X[blockIdx.z];
    const int32_t *__restrict__ hw = ab.hw[blockIdx.z];
    const float *__restrict__ sum = ab.sum[blockIdx.z];
    float *__restrict__ out = ab.out[blockIdx.z];
    const long o = (long)blockIdx.x * kBlock + threadIdx.x;
    const int RS = g.R * g.S, CRS = g.C * RS;
    if (o >= (long)g.K * CRS) return;
    const int k = (int)(o / CRS), j = (int)(o % CRS);
    const int c = j / RS, r = (j % RS) / g.S, s = j % g.S;
    const int n_begin = blockIdx.y * chunk_n;
    const int n_end = n_begin + chunk_n < g.N ? n_begin + chunk_n : g.N;
    float acc = 0.f;
#pragma unroll 4
    for (int n = n_begin; n < n_end; ++n) {
        const int p = hw[(long)n * g.K + k];
        const float sv = sum[(long)n * g.K + k];
        const int ih = (p >> 16) * g.sh + r - g.ph, iw = (p & 0xffff) * g.sw + s - g.pw;
        if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
            const long xi = (((long)n * g.C + c) * g.H + ih) * g.W + iw;
            const float xv = BF16 ? bf16_bits_to_float(((const uint16_t *)X)[xi]) : ((const float *)X)[xi];
            acc = fmaf(sv, xv, acc);
        }
    }
    out[(long)blockIdx.y * g.K * CRS + o] = acc * scale;
}

// ------------------------------------------------------------------------------------
// gather, LDS form (3x3 filters): used when the K patches of an image cover its input
// planes many times over (small planes, many output channels).  A workgroup (8 wavefronts) owns
// 8*M output channels x 64 input channels and walks a chunk of the batch in groups of
// `nb` images; every wavefront handles M output channels with one input channel per
// lane and keeps its 9*M sums in registers.
//
// Per group the 64 input planes of the nb images are staged in LDS with a zero halo
// (the padding the taps can reach), so a patch is nine unconditional reads at
// window origin + r*WP + s; the halo is zeroed once, staging only writes the interior.
// The plane pitch is odd: 32 consecutive channels hit 32 banks.  Everything is
// software-pipelined one group ahead: the global loads of group g+1 (input planes, and
// the (row, col, S) of the group's nb*M maps, one per lane) are issued before group g
// is computed, and LDS is double-buffered so one barrier per group suffices.  The
// selected position and sum of a map are moved to scalar registers with v_readlane, so
// the window origin is scalar arithmetic and S is a scalar multiplier.
// ------------------------------------------------------------------------------------
constexpr int kGatherCT = 64;
constexpr int kGatherBlock = 512;   // 8 wavefronts: two per SIMD, so one hides the LDS and scalar latencies of the other
constexpr int kGatherSlots = 4;      // 16-byte loads per thread and group (registers that stay live under the patch loop)
constexpr size_t kGatherLds = 64 * 1024;

template <bool BF16> struct Raw4 { typedef float4 type; };
template <> struct Raw4<true> { typedef uint2 type; };   // 4 bf16

struct GatherParams {
    int ctiles, nb, chunk_n;
    int wp, pitch;                   // haloed row pitch, LDS pitch of a haloed plane (odd)
    FastDiv d_hw4, d_w;
    float scale;
    int tk;                          // top-k form: kept positions per map (hw holds tk entries per map) ...
    float inv_k;                     // ... each weighted by sum / tk
};

// TOPK: every map contributes tk patches (its kept positions, hw[(n*K + k)*tk + t]) with weight sum/tk
// instead of one with weight sum; a group is then limited to nb*M*tk <= 64 (position, weight) pairs.
// (bx, by, bz): the workgroup's tile (channel tile fastest), batch chunk and problem
template <bool BF16, int M, bool TOPK>
__device__ __forceinline__ void gather_lds_body(const ApproxBatch &ab, const Geometry &g, const GatherParams &gp,
                                                float *__restrict__ xs, int bx, int by, int bz)
{
    const void *__restrict__ X = ab.X[bz];
    const int32_t *__restrict__ hw = ab.hw[bz];
    const float *__restrict__ sum = ab.sum[bz];
    float *__restrict__ out = ab.out[bz];
    typedef typename Raw4<BF16>::type raw4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ctile = bx % gp.ctiles, ktile = bx / gp.ctiles;
    const int c0 = ctile * kGatherCT;
    const int k_base = ktile * (kGatherBlock / 64 * M) + wave * M;
    const int HW = g.H * g.W, hw4 = HW >> 2;
    const int nb = gp.nb, pitch = gp.pitch, WP = gp.wp;
    const int n_begin = by * gp.chunk_n;
    const int n_end = n_begin + gp.chunk_n < g.N ? n_begin + gp.chunk_n : g.N;
    const int cvalid = g.C - c0 < kGatherCT ? g.C - c0 : kGatherCT;   // channels of this tile inside X
    const int run4 = cvalid * hw4;                        // 16-byte pieces per image
    const int buf_floats = nb * kGatherCT * pitch;
    FastDiv d_run4;                                       // run4 differs for the last channel tile
    d_run4.d = run4;
    d_run4.m = run4 > 1 ? (uint32_t)((1ull << 32) / (uint32_t)run4) + 1u : 0u;
    d_run4.one = run4 > 1 ? 0u : 0xffffffffu;

    for (int e = tid; e < 2 * buf_floats; e += kGatherBlock) xs[e] = 0.f;   // halo (and everything else) = 0

    float acc[M][9];
#pragma unroll
    for (int j = 0; j < M; ++j)
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[j][t] = 0.f;

    raw4 xr[kGatherSlots];
    int hw_next = 0;
    float sv_next = 0.f;

    // This thread's staging slots, decoded once: slot u is the 16-byte piece e = tid + u * kGatherBlock of a group
    // (image e / run4 of the group, then channel, then four consecutive elements of the plane).
    //   slot_src: element offset of the piece from the first image of a group
    //   slot_dst: float index of its first element in a window buffer | image within the group << 20; -1 = none
    // The four elements go to dst + {0,1,2,3} when a plane row holds a multiple of four (rowmode 0), to
    // dst + {0,1,WP,WP+1} for rows of two (rowmode 1); any other width takes the divisions per element (rowmode 2).
    const int rowmode = g.W % 4 == 0 ? 0 : (g.W == 2 ? 1 : 2);
    uint32_t slot_src[kGatherSlots];
    int slot_dst[kGatherSlots];
#pragma unroll
    for (int u = 0; u < kGatherSlots; ++u) {
        const int e = tid + u * kGatherBlock;
        slot_src[u] = 0; slot_dst[u] = -1;
        if (e < nb * run4) {
            uint32_t n_l, rem, c_l, q4, ih, iw;
            d_run4.divmod(e, n_l, rem);
            gp.d_hw4.divmod(rem, c_l, q4);
            gp.d_w.divmod(q4 * 4, ih, iw);
            slot_src[u] = n_l * (uint32_t)(g.C * HW) + rem * 4;
            slot_dst[u] = (int)((n_l * kGatherCT + c_l) * pitch + (g.ph + ih) * WP + g.pw + iw) | (int)(n_l << 20);
        }
    }

    // (position, sum) of the maps, one per lane, for a block of blk_groups groups at a time (not per group: with
    // one image of 8x8 planes per group, two loads per wavefront and group that serve two lanes each cost as much
    // of the load path as the planes themselves): lane l holds map (image b0 + l / M, channel k_base + l % M).
    const int blk_groups = (64 / M) / nb;                  // nb <= 64 / M
    const int blk_images = blk_groups * nb;
    int hw_blk = 0, hw_blk_next = 0;
    float sv_blk = 0.f, sv_blk_next = 0.f;
    auto prefetch_maps = [&](int b0) {
        const int n = b0 + lane / M, k = k_base + lane % M;
        const bool ok = lane < blk_images * M && n < n_end && k < g.K;
        hw_blk_next = ok ? hw[(long)n * g.K + k] : 0;
        sv_blk_next = ok ? sum[(long)n * g.K + k] : 0.f;
    };
    // Issue the loads of slots [U0, U0 + UN) of the group starting at image n0 (registers only).  ALWAYS: every
    // slot loads -- one without a piece re-reads the group's first piece -- so that the number of loads in flight
    // is fixed and a later wait can name exactly the older ones.
    auto prefetch_slots = [&](int n0, auto u0_c, auto un_c, auto always_c) {
        constexpr int U0 = decltype(u0_c)::value, UN = decltype(un_c)::value;
        constexpr bool ALWAYS = decltype(always_c)::value;
        const int nb_cur = n_end - n0 < nb ? n_end - n0 : nb;
        const long base = ((long)n0 * g.C + c0) * HW;
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const bool live = slot_dst[u] >= 0 && (slot_dst[u] >> 20) < nb_cur;
            if (ALWAYS || live) {
                const long src = base + (live ? slot_src[u] : 0u);
                xr[U0 + u] = BF16 ? *(const raw4 *)((const uint16_t *)X + src) : *(const raw4 *)((const float *)X + src);
            }
        }
    };
    // top-k form: the kept positions and weights of the group's maps, one per lane
    auto prefetch_topk = [&](int n0) {
        const int per_img = M * gp.tk;
        const int n = n0 + lane / per_img, q = lane % per_img;
        const int k = k_base + q / gp.tk, t = q % gp.tk;
        const bool ok = lane < nb * per_img && n < n_end && k < g.K;
        hw_next = ok ? hw[((long)n * g.K + k) * gp.tk + t] : 0;
        sv_next = ok ? sum[(long)n * g.K + k] * gp.inv_k : 0.f;
    };
    // registers of slots [U0, U0 + UN) -> LDS (interior of the haloed planes)
    auto commit_slots = [&](int nb_cur, float *buf, auto u0_c, auto un_c) {
        constexpr int U0 = decltype(u0_c)::value, UN = decltype(un_c)::value;
#pragma unroll
        for (int u = 0; u < UN; ++u)
            if (slot_dst[u] >= 0 && (slot_dst[u] >> 20) < nb_cur) {
                float v[4];
                if (BF16) {
                    const uint2 r = *(const uint2 *)&xr[U0 + u];
                    v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
                    v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
                } else {
                    const float4 r = *(const float4 *)&xr[U0 + u];
                    v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
                }
                float *dst = buf + (slot_dst[u] & 0xfffff);
                if (rowmode == 0) {
                    dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
                } else if (rowmode == 1) {
                    dst[0] = v[0]; dst[1] = v[1]; dst[WP] = v[2]; dst[WP + 1] = v[3];
                } else {
                    // dst is the cell of the piece's first element: walk on from its column
                    const int cell0 = (slot_dst[u] & 0xfffff) % pitch;          // offset inside the haloed plane
                    int iw = (cell0 % WP) - g.pw;
                    float *q = dst;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        *q = v[i];
                        if (++iw == g.W) { iw = 0; q += WP - g.W + 1; } else ++q;
                    }
                }
            }
    };
    // The patches of one group out of window buffer buf: one per (image, output channel) pair t = n_l * M + j, nine
    // LDS reads and nine multiply-adds each.  The reads of pair t + 1 are issued before the multiply-adds of pair t
    // (two register sets, alternating), so a wavefront always has a patch in flight behind the one it is adding.
    // No branches inside the loop: a pair index beyond the group re-reads the last pair and adds it with weight
    // zero.  slot0: lane that holds the group's first map in hw_blk / sv_blk.
    auto gather_group = [&](const float *buf, int nb_cur, int slot0) {
        if (lane >= cvalid || nb_cur <= 0) return;
        const float *plane = buf + lane * pitch;
        const int T = nb_cur * M;
        float v[2][9];
        auto issue = [&](int t, float (&dst)[9]) {
            t = t < T ? t : T - 1;
            const int p = __builtin_amdgcn_readlane(hw_blk, slot0 + t);
            const float *win = plane + (t / M) * (kGatherCT * pitch) + (p >> 16) * g.sh * WP + (p & 0xffff) * g.sw;
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s3 = 0; s3 < 3; ++s3) dst[r * 3 + s3] = win[r * WP + s3];
        };
        auto add = [&](int t, int j, const float (&src)[9]) {
            float sv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sv_blk), slot0 + (t < T ? t : T - 1)));
            sv = t < T ? sv : 0.f;
#pragma unroll
            for (int e = 0; e < 9; ++e) acc[j][e] = fmaf(sv, src[e], acc[j][e]);
        };
        constexpr int U = M == 1 ? 2 : M;               // pairs per trip: the output channel t % M and the register set
        issue(0, v[0]);                                 // t & 1 of a pair are compile-time constants
        for (int t0 = 0; t0 < T; t0 += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                issue(t0 + u + 1, v[(u + 1) & 1]);
                add(t0 + u, u % M, v[u & 1]);
            }
        }
    };
    // the (position, sum) block of the group that starts at image n0; returns the lane of the group's first map
    int gi_blk = 0;                                        // the group's number within its block of maps
    auto maps_for_group = [&](int n0) {
        if (gi_blk == blk_groups) gi_blk = 0;
        if (gi_blk == 0) {
            // a new block: take over what was requested a block ago (opaque moves: the wait sits here), request the next
            asm volatile("v_mov_b32 %0, %1" : "=v"(hw_blk) : "v"(hw_blk_next));
            asm volatile("v_mov_b32 %0, %1" : "=v"(sv_blk) : "v"(sv_blk_next));
            if (n0 + blk_images < n_end) prefetch_maps(n0 + blk_images);
        }
        return gi_blk++ * nb * M;
    };
    using ic0 = std::integral_constant<int, 0>;
    using ic2 = std::integral_constant<int, 2>;
    using icS = std::integral_constant<int, kGatherSlots>;

    FTRACE(0);
    long long t_stage = 0, t_loop = 0, t_mark = FTRACE_CLOCK();
    // A group that needs at most two staging slots per thread (one image of 8x8 planes) is far shorter than a load
    // takes to arrive: the four slot registers then hold TWO groups, the loads of group g + 2 being issued while
    // group g is computed.  Both groups of a trip run unconditionally (a group beyond the chunk commits and adds
    // nothing) and every slot loads, so the wait before a commit names exactly its own loads.
    const bool two_deep = !TOPK && kGatherSlots == 4 && nb * kGatherCT * hw4 <= 2 * kGatherBlock;
    if (two_deep) {
        prefetch_maps(n_begin);
        prefetch_slots(n_begin, ic0(), ic2(), std::true_type());
        prefetch_slots(n_begin + nb < n_end ? n_begin + nb : n_end - 1, ic2(), ic2(), std::true_type());
        __syncthreads();                                   // the zero fill is complete
        auto one_group = [&](int n0, auto set_c) {
            constexpr int SET = decltype(set_c)::value;
            const int nb_cur = n0 >= n_end ? 0 : (n_end - n0 < nb ? n_end - n0 : nb);
            float *buf = xs + SET * buf_floats;
            const int slot0 = nb_cur > 0 ? maps_for_group(n0) : 0;
            commit_slots(nb_cur, buf, std::integral_constant<int, 2 * SET>(), ic2());
            __syncthreads();
            prefetch_slots(n0 + 2 * nb < n_end ? n0 + 2 * nb : n_end - 1, std::integral_constant<int, 2 * SET>(), ic2(), std::true_type());
            { const long long now = FTRACE_CLOCK(); t_stage += now - t_mark; t_mark = now; }
            gather_group(buf, nb_cur, slot0);
            { const long long now = FTRACE_CLOCK(); t_loop += now - t_mark; t_mark = now; }
        };
        for (int n0 = n_begin; n0 < n_end; n0 += 2 * nb) {
            one_group(n0, ic0());
            one_group(n0 + nb, std::integral_constant<int, 1>());
        }
    } else {
        if (TOPK) prefetch_topk(n_begin); else prefetch_maps(n_begin);
        prefetch_slots(n_begin, ic0(), icS(), std::false_type());
        int parity = 0;
        for (int n0 = n_begin; n0 < n_end; n0 += nb, parity ^= 1) {
            const int nb_cur = n_end - n0 < nb ? n_end - n0 : nb;
            float *buf = xs + parity * buf_floats;
            const int slot0 = TOPK ? 0 : maps_for_group(n0);
            if (n0 == n_begin) __syncthreads();           // the zero fill is complete
            commit_slots(nb_cur, buf, ic0(), icS());
            // Copy through an opaque move: it makes the wait for these two loads happen here, where
            // they have long arrived, instead of at their first use below, after the next group's
            // loads have been issued (the memory counter is in-order: waiting there would drain those).
            int hw_cur;
            float sv_cur;
            asm volatile("v_mov_b32 %0, %1" : "=v"(hw_cur) : "v"(hw_next));
            asm volatile("v_mov_b32 %0, %1" : "=v"(sv_cur) : "v"(sv_next));
            __syncthreads();
            if (n0 + nb < n_end) {
                if (TOPK) prefetch_topk(n0 + nb);
                prefetch_slots(n0 + nb, ic0(), icS(), std::false_type());
            }
            { const long long now = FTRACE_CLOCK(); t_stage += now - t_mark; t_mark = now; }
            if (!TOPK) gather_group(buf, nb_cur, slot0);
            { const long long now = FTRACE_CLOCK(); t_loop += now - t_mark; t_mark = now; }
            if (lane < cvalid && TOPK) {
                const float *plane = buf + lane * pitch;
                for (int n_l = 0; n_l < nb_cur; ++n_l, plane += kGatherCT * pitch) {
#pragma unroll
                    for (int j = 0; j < M; ++j) {
                        for (int t = 0; t < gp.tk; ++t) {
                            const int slot = (n_l * M + j) * gp.tk + t;
                            const int p = __builtin_amdgcn_readlane(hw_cur, slot);
                            const float sv = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, sv_cur), slot));
                            const float *win = plane + (p >> 16) * g.sh * WP + (p & 0xffff) * g.sw;   // window origin
#pragma unroll
                            for (int r = 0; r < 3; ++r) {
                                const float *row = win + r * WP;
#pragma unroll
                                for (int s = 0; s < 3; ++s) acc[j][r * 3 + s] = fmaf(sv, row[s], acc[j][r * 3 + s]);
                            }
                        }
                    }
                }
            }
        }
    }
    FTRACE_SET(1, t_stage); FTRACE_SET(2, t_loop);
    if (lane < cvalid) {
        float *o = out + (long)by * g.K * g.C * 9;
#pragma unroll
        for (int j = 0; j < M; ++j) {
            const int k = k_base + j;
            if (k >= g.K) continue;
#pragma unroll
            for (int t = 0; t < 9; ++t) o[((long)k * g.C + c0 + lane) * 9 + t] = acc[j][t] * gp.scale;
        }
    }
    FTRACE(3);
}

template <bool BF16, int M, bool TOPK = false>
__global__ __launch_bounds__(kGatherBlock, 4) void approx_gather_lds3x3(ApproxBatch ab, Geometry g, GatherParams gp)
{
    extern __shared__ float xs[];                         // [2][nb][64][pitch]
    gather_lds_body<BF16, M, TOPK>(ab, g, gp, xs, blockIdx.x, blockIdx.y, blockIdx.z);
}

// The gathers of several layer groups of a schedule run as one grid (the groups' ramps and tails overlap instead
// of adding up): a workgroup looks its group up in a table in the kernel arguments, read in place (see the
// fused form's multi-group launch for why).
constexpr int kGatherMultiMax = 6;
struct GatherGroup {
    ApproxBatch ab;
    Geometry g;
    GatherParams gp;
    int gx, gy;                      // tiles and batch chunks of the group's own grid (z = problems)
};
struct GatherMulti {
    int n;
    int begin[kGatherMultiMax + 1];  // first workgroup of each group; begin[n] = grid size
    GatherGroup grp[kGatherMultiMax];
};

template <bool BF16, int M>
__global__ __launch_bounds__(kGatherBlock, 4) void approx_gather_lds_multi(const GatherMulti)
{
    extern __shared__ float xs[];
    const GatherMulti *mp = (const GatherMulti *)__builtin_amdgcn_kernarg_segment_ptr();
    const int n = mp->n;
    int gi = 0;
    for (int i = 1; i < n; ++i) gi += (int)blockIdx.x >= mp->begin[i];
    const GatherGroup &G = mp->grp[gi];
    const int linear = (int)blockIdx.x - mp->begin[gi];
    const int bx = linear % G.gx, rest = linear / G.gx;
    gather_lds_body<BF16, M, false>(G.ab, G.g, G.gp, xs, bx, rest % G.gy, rest / G.gy);
}

// ------------------------------------------------------------------------------------
// fused form (large maps, few output channels: the regime of the direct gather).  One
// workgroup = one output channel k and one chunk of the batch; each wavefront walks its
// images: it scans the map dY[n,k,:,:] (16-byte pieces, all 64 lanes; the next image's map
// is already in flight), reduces (|v| bits, position) and the sum across the wavefront,
// and immediately gathers the C*R*S patch the selected position sees, one or more dW
// entries per lane, accumulating in registers over its images.  The four wavefronts'
// sums are added through LDS.  Position and sum never travel through memory; dY is read
// exactly once from HBM.  Requires Ho*Wo <= 1024 (a multiple of 4); the C*R*S entries of an output channel are
// cut into slices of 576, one workgroup each (up to four: the slices of a channel scan the same maps, the
// later ones out of L2).
// ------------------------------------------------------------------------------------
constexpr int kFusedJ = 9;       // dW entries of one output channel per lane
constexpr int kFusedV = 4;       // 4-element pieces of one map per lane
constexpr int kFusedSlices = 4;  // workgroups that share the entries of one output channel (C*R*S up to 4 * 576)

// slices of kFusedJ * 64 entries that the C*R*S entries of one output channel are cut into
static inline int fused_slices(const Geometry &g) { return (int)((g.crs() + 64 * kFusedJ - 1) / (64 * kFusedJ)); }

struct FusedParams {
    int chunk_n;
    float scale;
    FastDiv d_rs, d_s, d_wo;
    int32_t *flat_out;           // optional user outputs (single-problem launches only)
    float *sum_out;
    int dw_layout;               // channel-last form only: where the result goes (WGRAD_DW_*)
    int tk;                      // top-k form only: kept positions per map, each weighted by sum * inv_k
    float inv_k;
    int nslice;                  // workgroups per output channel, each owning kFusedJ * 64 of its C*R*S entries
    int slice_major;             // numbering of the nslice * K workgroups of a chunk: all K of slice 0 first (1), or the slices of a channel side by side (0)
    int rows3;                   // filter-row form (fp32, NCHW, S = 3): (channel, row) pairs per lane, 1..3; 0 = element form
    FastDiv d_r;
};

// Whether the filter-row form takes the shape, and with how many pairs per lane: width-3 filters on fp32 NCHW
// input whose patches overhang a row of X by at most one column on either side.
static inline int fused_rows3(const Geometry &g)
{
    if (g.bf16 || g.S != 3 || g.W < 3 || g.pw > 1 || g.R > 63) return 0;
    if ((long)(g.Wo - 1) * g.sw - g.pw + 3 - g.W > 1) return 0;
    const long cr = (long)g.C * g.R;
    const long per_slice = cr < kFusedJ * 64 / 3 ? cr : kFusedJ * 64 / 3;
    return (int)((per_slice + 63) / 64);
}

// linear: the workgroup's number among the nk * nchunks * nprob of its group
//
// NHWC = true is the layout of the paper's own kernel (Section 2.4): X[n,h,w,c], so that a patch is R
// rows of S*C contiguous values and consecutive lanes read consecutive channels; the entries of one
// output channel are then numbered (r, s, c) and fp.d_rs divides by C.
// TOPK = true keeps fp.tk positions per map: the scan is repeated with "largest rank key below the last one
// found" (keys (|v| bits << 32) | ~position are unique within a map), every kept position's patch enters
// the same one-step-delayed accumulation with weight sum / tk.
// V, FULLMAP: a map is V 16-byte pieces per lane; FULLMAP says that every lane holds all V of them (maps of
// exactly 256*V positions), which leaves the image loop free of conditional loads and of branches.
// ROWS (maps of up to 64 positions, V = 1): a map fills at most one row of 16 lanes, so a wavefront scans the
// maps of four images at once, one per row, and reduces them with the row steps of the scans alone; the
// four patches are then gathered one after the other as before.  The scan and the reductions, half of the
// vector instructions of a small map, are shared by four maps.
template <bool BF16, bool NHWC, bool TOPK, int V, bool FULLMAP, bool ROWS = false>
__device__ __forceinline__ void fused_body(const ApproxBatch &ab, const Geometry &g, const FusedParams &fp,
                                           float (&red)[4][kFusedJ * 64], int linear, int nk, int nchunks, int nprob)
{
    typedef typename Raw4<BF16>::type raw4;
    constexpr int ESZ = BF16 ? 2 : 4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // The K workgroups of one (problem, batch chunk) read the same input planes: number the workgroups so
    // that they sit on one XCD and find each other's planes in its L2.
    // nk = K * fp.nslice.  Slice-major numbering: the K workgroups of one slice are neighbours, so an XCD that runs a
    // slice needs only that slice's 64 input channels of the chunk in its L2 (the maps are then fetched once per
    // slice: measured 93 -> 64 MB on 128->128 @ 16x16, N = 128, against the slices of a channel side by side).
    const int logical = xcd_contiguous_id(linear, nk * nchunks * nprob);
    const int kk = logical % nk;
    const int k = fp.slice_major ? kk % g.K : kk / fp.nslice;
    const int j_base = (fp.slice_major ? kk / g.K : kk - k * fp.nslice) * (kFusedJ * 64);
    const bool first_slice = j_base == 0;                  // writes the optional position / sum outputs
    const int by = (logical / nk) % nchunks, bz = logical / (nk * nchunks);
    const char *__restrict__ X = (const char *)ab.X[bz];
    const char *__restrict__ dY = (const char *)ab.dY[bz];
    float *__restrict__ out = ab.out[bz];
    const int L = g.Ho * g.Wo, RS = g.R * g.S, CRS = g.C * RS, HW = g.H * g.W;
    const int n_begin = by * fp.chunk_n;
    const int n_end = n_begin + fp.chunk_n < g.N ? n_begin + fp.chunk_n : g.N;

    // the dW entries j = lane + 64*jj of channel k that this lane accumulates
    // xo: element offset of the entry's tap from the patch origin (bits 0-23) and the tap's number r*S + s
    // (bits 24-29); an entry beyond C*R*S has offset 0 and tap number 63, which no filter of the shapes
    // this form takes has (R*S <= 63)
    int xo[kFusedJ];
    float acc[kFusedJ];
#pragma unroll
    for (int jj = 0; jj < kFusedJ; ++jj) {
        const int j = j_base + lane + 64 * jj;
        uint32_t c, tap, r, s2;
        if (NHWC) fp.d_rs.divmod(j, tap, c);
        else      fp.d_rs.divmod(j, c, tap);
        fp.d_s.divmod(tap, r, s2);
        const uint32_t off = NHWC ? (r * g.W + s2) * g.C + c : c * HW + r * g.W + s2;
        xo[jj] = j < CRS ? (int)(off | tap << 24) : (int)(63u << 24);
        acc[jj] = 0.f;
    }

    float x_pend[kFusedJ], S_pend = 0.f;       // patch and sum of the previous image, not yet accumulated
#pragma unroll
    for (int jj = 0; jj < kFusedJ; ++jj) x_pend[jj] = 0.f;
    // one map buffer: the next image's map is requested as soon as the scan has consumed this one's, and
    // arrives under the butterfly, the accumulation and the patch request
    raw4 cur[V];
    auto load_map = [&](int n, raw4 (&m)[V]) {
        if (ROWS) {                            // row r of the wavefront: image n + 4r
            const int nr = n + 4 * (lane >> 4), e = (lane & 15) * 4;
            if (nr < n_end && e < L) m[0] = *(const raw4 *)(dY + (((long)nr * g.K + k) * L + e) * ESZ);
            return;
        }
        const char *base = dY + ((long)n * g.K + k) * L * ESZ;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int e = (lane + 64 * v) * 4;
            if (FULLMAP || e < L) m[v] = *(const raw4 *)(base + (long)e * ESZ);
        }
    };
    // the patch requested one step ago has had a whole scan to arrive: accumulate it (the loaded values are
    // touched only here, so the wait for them sits here and not behind the request)
    uint32_t pend_inside = 0;                  // bit jj: entry jj of the pending patch lies inside X
    bool pend_whole = true;                    // wavefront-uniform: the pending patch lies inside X entirely
    auto accumulate_pending = [&]() {
        if (pend_whole) {
#pragma unroll
            for (int jj = 0; jj < kFusedJ; ++jj)
                acc[jj] = fmaf(S_pend, BF16 ? __uint_as_float(__float_as_uint(x_pend[jj]) << 16) : x_pend[jj], acc[jj]);
        } else {
#pragma unroll
            for (int jj = 0; jj < kFusedJ; ++jj)
                acc[jj] = fmaf(S_pend, (pend_inside >> jj & 1) ? (BF16 ? __uint_as_float(__float_as_uint(x_pend[jj]) << 16) : x_pend[jj]) : 0.f,
                               acc[jj]);
        }
    };
    // request the patch of position pos of image n; it is accumulated one step later.  The kernel is bound
    // by the number of vector instructions per image, so the common case -- a patch that lies inside X
    // entirely, a wavefront-uniform test -- is one add and one load per entry; only patches that reach
    // into the padding pay for per-tap bounds.  Every lane loads unconditionally in both cases (a tap
    // outside X, or an entry beyond C*R*S, reads a valid element that is not used), so there are no
    // branches around the loads and all nine are in flight together.  Offsets are relative to the image
    // start, a scalar base.
    auto request_patch = [&](int n, int pos) {
        uint32_t h, w;
        fp.d_wo.divmod(pos, h, w);
        const int ihb = (int)h * g.sh - g.ph, iwb = (int)w * g.sw - g.pw;
        const char *Ximg = X + (long)n * g.C * HW * ESZ;
        const int origin = (ihb * g.W + iwb) * (NHWC ? g.C : 1);      // may be negative; a tap inside X is not
        pend_whole = ihb >= 0 && ihb + g.R <= g.H && iwb >= 0 && iwb + g.S <= g.W;
        if (pend_whole) {
#pragma unroll
            for (int jj = 0; jj < kFusedJ; ++jj) {
                const uint32_t off = (uint32_t)(origin + (xo[jj] & 0xffffff)) * ESZ;
                if (BF16) x_pend[jj] = __uint_as_float((uint32_t)*(const uint16_t *)(Ximg + off));   // widened when used
                else      x_pend[jj] = *(const float *)(Ximg + off);
            }
        } else {
            // which taps lie inside X depends on the position alone: one bit per tap number, built on the
            // scalar unit from the valid tap rows [r_lo, r_hi) and columns [s_lo, s_hi)
            const int r_lo = ihb < 0 ? -ihb : 0, r_hi = g.H - ihb < g.R ? g.H - ihb : g.R;
            const int s_lo = iwb < 0 ? -iwb : 0, s_hi = g.W - iwb < g.S ? g.W - iwb : g.S;
            unsigned long long taps = 0;
            if (s_hi > s_lo) {
                const unsigned long long cols = ((1ull << s_hi) - 1) & ~((1ull << s_lo) - 1);
                for (int r = r_lo; r < r_hi; ++r) taps |= cols << (r * g.S);
            }
            pend_inside = 0;
#pragma unroll
            for (int jj = 0; jj < kFusedJ; ++jj) {
                const uint32_t inside = (uint32_t)(taps >> ((uint32_t)xo[jj] >> 24)) & 1u;
                const uint32_t off = inside ? (uint32_t)(origin + (xo[jj] & 0xffffff)) * ESZ : 0u;
                pend_inside |= inside << jj;
                if (BF16) x_pend[jj] = __uint_as_float((uint32_t)*(const uint16_t *)(Ximg + off));
                else      x_pend[jj] = *(const float *)(Ximg + off);
            }
        }
    };
    FTRACE(1);
    if (n_begin + wave < n_end) load_map(n_begin + wave, cur);
    // Pass the first map through opaque moves: the wait for it then sits here, and the loop is entered with
    // no load pending on these registers.  Otherwise the wait the compiler places before the scan must
    // cover this first load on the entry path, and (the memory counter being in-order) it would then also
    // drain the previous image's patch loads in every iteration.
#pragma unroll
    for (int v = 0; v < V; ++v) {
        uint32_t *w = (uint32_t *)&cur[v];
#pragma unroll
        for (int i = 0; i < (int)(sizeof(raw4) / 4); ++i) asm volatile("v_mov_b32 %0, %1" : "=v"(w[i]) : "v"(w[i]));
    }
    for (int n = n_begin + wave; n < n_end; n += ROWS ? 16 : 4) {
        if (ROWS) {
            const int e = (lane & 15) * 4;
            const bool have = n + 4 * (lane >> 4) < n_end && e < L;
            uint32_t best_key = 0, best_pos = e;
            float sum = 0.f;
            if (have) {
                uint32_t bits[4];
                if (BF16) {
                    const uint2 r2 = *(const uint2 *)&cur[0];
                    bits[0] = r2.x << 16; bits[1] = r2.x & 0xffff0000u; bits[2] = r2.y << 16; bits[3] = r2.y & 0xffff0000u;
                } else {
                    const uint4 r4 = *(const uint4 *)&cur[0];
                    bits[0] = r4.x; bits[1] = r4.y; bits[2] = r4.z; bits[3] = r4.w;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t key = mag_key<BF16>(bits[i]);
                    if (key > best_key) { best_key = key; best_pos = e + i; }
                    sum += __uint_as_float(bits[i]);
                }
            }
            if (n + 16 < n_end) load_map(n + 16, cur);
            const uint32_t rmax = row_max_u32(best_key);
            const float rsum = row_sum_f32(sum);
            uint32_t kmax[4];
            float S4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                kmax[r] = (uint32_t)__builtin_amdgcn_readlane((int)rmax, 16 * r + 15);
                S4[r] = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(rsum), 16 * r + 15));
            }
            // the lowest lane of a row that holds the row's maximum holds its lowest position: lanes hold
            // ascending positions, and a lane keeps the first of equal values
            const uint32_t mine = lane < 32 ? (lane < 16 ? kmax[0] : kmax[1]) : (lane < 48 ? kmax[2] : kmax[3]);
            const unsigned long long eq = __ballot(have && best_key == mine);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int nr = n + 4 * r;
                if (nr >= n_end) break;                              // wavefront-uniform
                const uint32_t sub = (uint32_t)(eq >> (16 * r)) & 0xffffu;      // not zero: lane 0 of the row has data
                const int pos = __builtin_amdgcn_readlane((int)best_pos, 16 * r + __builtin_ctz(sub));
                if (lane == 0 && first_slice) {
                    if (fp.flat_out) fp.flat_out[(long)nr * g.K + k] = pos;
                    if (fp.sum_out) fp.sum_out[(long)nr * g.K + k] = S4[r];
                }
                accumulate_pending();
                request_patch(nr, pos);
                S_pend = S4[r];
            }
            continue;
        }
        if (TOPK) {
            float sum = 0.f, S = 0.f;
            unsigned long long below = ~0ull;
            for (int t = 0; t < fp.tk; ++t) {
                unsigned long long best = 0ull;          // lanes that hold nothing lose every comparison
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const int e = (lane + 64 * v) * 4;
                    if (FULLMAP || e < L) {
                        uint32_t bits[4];
                        if (BF16) {
                            const uint2 r2 = *(const uint2 *)&cur[v];
                            bits[0] = r2.x << 16; bits[1] = r2.x & 0xffff0000u; bits[2] = r2.y << 16; bits[3] = r2.y & 0xffff0000u;
                        } else {
                            const uint4 r4 = *(const uint4 *)&cur[v];
                            bits[0] = r4.x; bits[1] = r4.y; bits[2] = r4.z; bits[3] = r4.w;
                        }
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            unsigned long long pk = ((unsigned long long)mag_key<BF16>(bits[i]) << 32) | (uint32_t)~(uint32_t)(e + i);
                            pk = pk < below ? pk : 0ull;
                            best = pk > best ? pk : best;
                            if (t == 0) sum += __uint_as_float(bits[i]);
                        }
                    }
                }
                uint32_t key_max, inv_pos_max;
                wave_max_pair((uint32_t)(best >> 32), (uint32_t)best, key_max, inv_pos_max);
                if (t == 0) S = wave_sum_f32(sum);
                const int pos = (int)~inv_pos_max;
                below = ((unsigned long long)key_max << 32) | inv_pos_max;
                if (lane == 0 && first_slice) {
                    if (fp.flat_out) fp.flat_out[((long)n * g.K + k) * fp.tk + t] = pos;
                    if (fp.sum_out && t == 0) fp.sum_out[(long)n * g.K + k] = S;
                }
                accumulate_pending();
                request_patch(n, pos);
                S_pend = S * fp.inv_k;
            }
            if (n + 4 < n_end) load_map(n + 4, cur);
            continue;
        }
        // ---- select: per-lane scan in ascending position, then a butterfly over the wavefront ----
        uint32_t best_key = 0, best_pos = 0;
        bool have = false;
        float sum = 0.f;
#pragma unroll
        for (int v = 0; v < V; ++v) {
            const int e = (lane + 64 * v) * 4;
            if (FULLMAP || e < L) {
                uint32_t bits[4];
                if (BF16) {
                    const uint2 r2 = *(const uint2 *)&cur[v];
                    bits[0] = r2.x << 16; bits[1] = r2.x & 0xffff0000u; bits[2] = r2.y << 16; bits[3] = r2.y & 0xffff0000u;
                } else {
                    const uint4 r4 = *(const uint4 *)&cur[v];
                    bits[0] = r4.x; bits[1] = r4.y; bits[2] = r4.z; bits[3] = r4.w;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t key = mag_key<BF16>(bits[i]);
                    if (!have || key > best_key) { best_key = key; best_pos = e + i; have = true; }
                    sum += __uint_as_float(bits[i]);
                }
            }
        }
        if (n + 4 < n_end) load_map(n + 4, cur);
        uint32_t key_max, inv_pos_max;
        wave_max_pair(have ? best_key : 0u, have ? ~best_pos : 0u, key_max, inv_pos_max);
        const int pos = (int)~inv_pos_max;
        const float S = wave_sum_f32(sum);
        if (lane == 0 && first_slice) {
            if (fp.flat_out) fp.flat_out[(long)n * g.K + k] = pos;
            if (fp.sum_out) fp.sum_out[(long)n * g.K + k] = S;
        }
        accumulate_pending();
        request_patch(n, pos);
        S_pend = S;
    }
    accumulate_pending();
    FTRACE(2);
    // ---- add the four wavefronts' sums and write this chunk's row of the result ----
#pragma unroll
    for (int jj = 0; jj < kFusedJ; ++jj) red[wave][jj * 64 + lane] = acc[jj];
    __syncthreads();
    float *o = out + ((long)by * g.K + k) * CRS;
    const int j_end = CRS - j_base < kFusedJ * 64 ? CRS - j_base : kFusedJ * 64;
    for (int jl = tid; jl < j_end; jl += kBlock) {
        const int j = j_base + jl;
        const float v = (red[0][jl] + red[1][jl] + red[2][jl] + red[3][jl]) * fp.scale;
        if (!NHWC || fp.dw_layout == WGRAD_DW_OHWI) {
            o[j] = v;
        } else {
            uint32_t tap, c;
            fp.d_rs.divmod(j, tap, c);
            if (fp.dw_layout == WGRAD_DW_HWIO) out[(long)by * g.K * CRS + (long)j * g.K + k] = v;
            else                               o[c * RS + tap] = v;
        }
    }
}


// ------------------------------------------------------------------------------------
// fused form, filter rows as the unit (fp32, NCHW, filters of width 3, one kept position per map).
// The three taps of a filter row are three consecutive input elements, i.e. ONE 12-byte load (global loads of
// several dwords need only 4-byte alignment), so a lane owns (channel, filter row) pairs -- J3 of them, pair
// q = lane + 64*jj of the slice -- instead of single entries: a third of the load instructions and address
// arithmetic of the element form, and no lane loads for entries beyond C*R*S.
// Columns: the 12 bytes are read at column cw = clamp(iwb, 0, W-3), always inside the row; a patch whose first
// (last) column lies in the padding is the same three registers used one tap to the right (left).  Which of the
// three cases applies is wavefront-uniform (it depends on the position alone).  Rows outside X: the lane reads
// a valid address instead and its weight is zero.
// The wavefront works in batches of B maps: scan B maps, request the next batch's maps, accumulate the B patches
// requested one batch ago, request this batch's B patches -- every load has a whole batch of work to arrive
// under, and B times as many bytes are in flight per wavefront as with one map at a time (the kernel was bound by
// memory latency, one patch in flight per wavefront, not by bandwidth).
// ------------------------------------------------------------------------------------
struct __attribute__((packed, aligned(4))) Row3 { float v[3]; };
constexpr int kPairsPerSlice = kFusedJ * 64 / 3;     // (channel, filter row) pairs of one slice of 576 entries

template <int V, bool FULLMAP, bool ROWS, int J3>
__device__ __forceinline__ void fused3_body(const ApproxBatch &ab, const Geometry &g, const FusedParams &fp,
                                            float (&red)[4][kFusedJ * 64], int linear, int nk, int nchunks, int nprob)
{
    constexpr int B = V == 1 ? 4 : 1;                      // maps per batch (ROWS: the four rows of one load)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int logical = xcd_contiguous_id(linear, nk * nchunks * nprob);
    const int kk = logical % nk;
    const int k = fp.slice_major ? kk % g.K : kk / fp.nslice, slice = fp.slice_major ? kk / g.K : kk - k * fp.nslice;
    const bool first_slice = slice == 0;
    const int by = (logical / nk) % nchunks, bz = logical / (nk * nchunks);
    const char *__restrict__ X = (const char *)ab.X[bz];
    const char *__restrict__ dY = (const char *)ab.dY[bz];
    float *__restrict__ out = ab.out[bz];
    const int L = g.Ho * g.Wo, CR = g.C * g.R, CRS = CR * 3, HW = g.H * g.W;
    const int n_begin = by * fp.chunk_n;
    const int n_end = n_begin + fp.chunk_n < g.N ? n_begin + fp.chunk_n : g.N;

    // slot jj: pair q = (c, r); xo = element offset of the pair's row from the patch origin, r in bits 24-29.
    // A slot beyond C*R duplicates pair (0, 0): its loads are valid, its sums are never written.
    int xo[J3];
    float acc[J3][3];
#pragma unroll
    for (int jj = 0; jj < J3; ++jj) {
        const int q = slice * kPairsPerSlice + lane + 64 * jj;
        uint32_t c, r;
        fp.d_r.divmod(q, c, r);
        xo[jj] = q < CR ? (int)((c * HW + r * g.W) | r << 24) : 0;
        acc[jj][0] = acc[jj][1] = acc[jj][2] = 0.f;
    }

    // pending batch: the patches requested one batch ago
    float x_pend[B][J3][3];
    float S_pend[B];
    int ihb_pend[B], shift_pend[B];
    bool whole_pend[B];
#pragma unroll
    for (int b = 0; b < B; ++b) {
        S_pend[b] = 0.f; ihb_pend[b] = 0; shift_pend[b] = 0; whole_pend[b] = true;
#pragma unroll
        for (int jj = 0; jj < J3; ++jj) x_pend[b][jj][0] = x_pend[b][jj][1] = x_pend[b][jj][2] = 0.f;
    }
    auto accumulate_pending = [&]() {
#pragma unroll
        for (int b = 0; b < B; ++b) {
#pragma unroll
            for (int jj = 0; jj < J3; ++jj) {
                float wl = S_pend[b], y0 = x_pend[b][jj][0], y1 = x_pend[b][jj][1], y2 = x_pend[b][jj][2];
                if (!whole_pend[b]) {                       // wavefront-uniform: the patch reaches into the padding
                    if ((uint32_t)(ihb_pend[b] + (int)((uint32_t)xo[jj] >> 24)) >= (uint32_t)g.H) wl = 0.f;
                    if (shift_pend[b] > 0)      { y2 = y1; y1 = y0; y0 = 0.f; }   // first column in the padding
                    else if (shift_pend[b] < 0) { y0 = y1; y1 = y2; y2 = 0.f; }   // last column in the padding
                }
                acc[jj][0] = fmaf(wl, y0, acc[jj][0]);
                acc[jj][1] = fmaf(wl, y1, acc[jj][1]);
                acc[jj][2] = fmaf(wl, y2, acc[jj][2]);
            }
        }
    };
    auto request_patch = [&](int b, int n, int pos, float S) {
        uint32_t h, w;
        fp.d_wo.divmod(pos, h, w);
        const int ihb = (int)h * g.sh - g.ph, iwb = (int)w * g.sw - g.pw;
        const int cw = iwb < 0 ? 0 : (iwb > g.W - 3 ? g.W - 3 : iwb);
        const char *Ximg = X + (long)n * g.C * HW * 4;
        const bool whole = ihb >= 0 && ihb + g.R <= g.H && cw == iwb;
        const int origin = ihb * g.W + cw;                  // may be negative when rows lie above X; a valid row's is not
        S_pend[b] = S; ihb_pend[b] = ihb; shift_pend[b] = cw - iwb; whole_pend[b] = whole;
        if (whole) {
#pragma unroll
            for (int jj = 0; jj < J3; ++jj) {
                const Row3 t = *(const Row3 *)(Ximg + (uint32_t)(origin + (xo[jj] & 0xffffff)) * 4u);
                x_pend[b][jj][0] = t.v[0]; x_pend[b][jj][1] = t.v[1]; x_pend[b][jj][2] = t.v[2];
            }
        } else {
#pragma unroll
            for (int jj = 0; jj < J3; ++jj) {
                const bool ok = (uint32_t)(ihb + (int)((uint32_t)xo[jj] >> 24)) < (uint32_t)g.H;
                const uint32_t off = ok ? (uint32_t)(origin + (xo[jj] & 0xffffff)) * 4u : 0u;
                const Row3 t = *(const Row3 *)(Ximg + off);
                x_pend[b][jj][0] = t.v[0]; x_pend[b][jj][1] = t.v[1]; x_pend[b][jj][2] = t.v[2];
            }
        }
    };

    // ---- maps: image n + 4*b of the batch starting at image n (this wavefront's images are n_begin + wave + 4*i) ----
    float4 cur[ROWS ? 1 : B][V];
    auto load_maps = [&](int n) {
        if (ROWS) {                                         // row b of the wavefront: image n + 4b, 16 lanes x 16 bytes
            const int nr = n + 4 * (lane >> 4), e = (lane & 15) * 4;
            if (nr < n_end && e < L) cur[0][0] = *(const float4 *)(dY + (((long)nr * g.K + k) * L + e) * 4);
            return;
        }
#pragma unroll
        for (int b = 0; b < B; ++b) {
            if (n + 4 * b >= n_end) break;                  // wavefront-uniform
            const char *base = dY + ((long)(n + 4 * b) * g.K + k) * L * 4;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const int e = (lane + 64 * v) * 4;
                if (FULLMAP || e < L) cur[b][v] = *(const float4 *)(base + (long)e * 4);
            }
        }
    };
    FTRACE(1);
    if (n_begin + wave < n_end) load_maps(n_begin + wave);
    // the first maps pass through opaque moves: the wait for them sits here, and the loop is entered with no load
    // pending on these registers (otherwise the wait before every scan would also drain the pending patches)
#pragma unroll
    for (int b = 0; b < (ROWS ? 1 : B); ++b)
#pragma unroll
        for (int v = 0; v < V; ++v) {
            uint32_t *wd = (uint32_t *)&cur[b][v];
#pragma unroll
            for (int i = 0; i < 4; ++i) asm volatile("v_mov_b32 %0, %1" : "=v"(wd[i]) : "v"(wd[i]));
        }
    for (int n = n_begin + wave; n < n_end; n += 4 * B) {
        int pos[B];
        float S[B];
        if (ROWS) {
            const int e = (lane & 15) * 4;
            const bool have = n + 4 * (lane >> 4) < n_end && e < L;
            uint32_t best_key = 0, best_pos = e;
            float sum = 0.f;
            if (have) {
                const uint4 r4 = *(const uint4 *)&cur[0][0];
                const uint32_t bits[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t key = mag_key<false>(bits[i]);
                    if (key > best_key) { best_key = key; best_pos = e + i; }
                    sum += __uint_as_float(bits[i]);
                }
            }
            const uint32_t rmax = row_max_u32(best_key);
            const float rsum = row_sum_f32(sum);
            uint32_t kmax[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                kmax[r] = (uint32_t)__builtin_amdgcn_readlane((int)rmax, 16 * r + 15);
                S[r] = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(rsum), 16 * r + 15));
            }
            // the lowest lane of a row that holds the row's maximum holds its lowest position
            const uint32_t mine = lane < 32 ? (lane < 16 ? kmax[0] : kmax[1]) : (lane < 48 ? kmax[2] : kmax[3]);
            const unsigned long long eq = __ballot(have && best_key == mine);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const uint32_t sub = (uint32_t)(eq >> (16 * r)) & 0xffffu;       // zero only for a row without an image
                pos[r] = __builtin_amdgcn_readlane((int)best_pos, 16 * r + (sub ? __builtin_ctz(sub) : 0));
            }
        } else {
#pragma unroll
            for (int b = 0; b < B; ++b) {
                uint32_t best_key = 0, best_pos = 0;
                bool have = false;
                float sum = 0.f;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const int e = (lane + 64 * v) * 4;
                    if (FULLMAP || e < L) {
                        const uint4 r4 = *(const uint4 *)&cur[b][v];
                        const uint32_t bits[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const uint32_t key = mag_key<false>(bits[i]);
                            if (!have || key > best_key) { best_key = key; best_pos = e + i; have = true; }
                            sum += __uint_as_float(bits[i]);
                        }
                    }
                }
                if (V == 1) {
                    // one piece per lane: lanes hold ascending positions, so the lowest lane that holds the
                    // maximum holds its lowest position
                    const uint32_t key_max = wave_max_u32(have ? best_key : 0u);
                    const unsigned long long eq = __ballot(have && best_key == key_max);
                    pos[b] = __builtin_amdgcn_readlane((int)best_pos, eq ? (int)__builtin_ctzll(eq) : 0);
                } else {
                    uint32_t key_max, inv_pos_max;
                    wave_max_pair(have ? best_key : 0u, have ? ~best_pos : 0u, key_max, inv_pos_max);
                    pos[b] = (int)~inv_pos_max;
                }
                S[b] = wave_sum_f32(sum);
            }
        }
        if (n + 4 * B < n_end) load_maps(n + 4 * B);
        accumulate_pending();
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const int nb = n + 4 * b;
            if (nb >= n_end) { S_pend[b] = 0.f; continue; }            // wavefront-uniform
            if (lane == 0 && first_slice) {
                if (fp.flat_out) fp.flat_out[(long)nb * g.K + k] = pos[b];
                if (fp.sum_out) fp.sum_out[(long)nb * g.K + k] = S[b];
            }
            request_patch(b, nb, pos[b], S[b]);
        }
    }
    accumulate_pending();
    FTRACE(2);
    // ---- add the four wavefronts' sums and write this chunk's row of the result ----
#pragma unroll
    for (int jj = 0; jj < J3; ++jj)
#pragma unroll
        for (int t = 0; t < 3; ++t) red[wave][(lane + 64 * jj) * 3 + t] = acc[jj][t];
    __syncthreads();
    const int j_base = slice * (kFusedJ * 64);
    float *o = out + ((long)by * g.K + k) * CRS;
    const int j_end = CRS - j_base < kFusedJ * 64 ? CRS - j_base : kFusedJ * 64;
    for (int jl = tid; jl < j_end; jl += kBlock)
        o[j_base + jl] = (red[0][jl] + red[1][jl] + red[2][jl] + red[3][jl]) * fp.scale;
}

template <int J3>
__device__ __forceinline__ void fused3_by_map(const ApproxBatch &ab, const Geometry &g, const FusedParams &fp,
                                              float (&red)[4][kFusedJ * 64], int linear, int nk, int nchunks, int nprob)
{
    const int L = g.Ho * g.Wo;
    if (L <= 64)        fused3_body<1, false, true, J3>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else if (L == 1024) fused3_body<4, true, false, J3>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else if (L == 256)  fused3_body<1, true, false, J3>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else if (L < 256)   fused3_body<1, false, false, J3>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else                fused3_body<kFusedV, false, false, J3>(ab, g, fp, red, linear, nk, nchunks, nprob);
}

__device__ __forceinline__ void fused3_dispatch(const ApproxBatch &ab, const Geometry &g, const FusedParams &fp,
                                                float (&red)[4][kFusedJ * 64], int linear, int nk, int nchunks, int nprob)
{
    if (fp.rows3 == 1)      fused3_by_map<1>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else if (fp.rows3 == 2) fused3_by_map<2>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else                    fused3_by_map<3>(ab, g, fp, red, linear, nk, nchunks, nprob);
}

// Picks the body for the map size: maps of exactly 1024 or 256 positions get the branch-free forms, maps of
// up to 64 positions the four-maps-per-wavefront form.
template <bool BF16, bool NHWC, bool TOPK>
__device__ __forceinline__ void fused_dispatch(const ApproxBatch &ab, const Geometry &g, const FusedParams &fp,
                                               float (&red)[4][kFusedJ * 64], int linear, int nk, int nchunks, int nprob)
{
    const int L = g.Ho * g.Wo;
    if (L <= 64 && !TOPK) fused_body<BF16, NHWC, false, 1, false, true>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else if (L == 1024) fused_body<BF16, NHWC, TOPK, 4, true>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else if (L == 256) fused_body<BF16, NHWC, TOPK, 1, true>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else if (L < 256)  fused_body<BF16, NHWC, TOPK, 1, false>(ab, g, fp, red, linear, nk, nchunks, nprob);
    else               fused_body<BF16, NHWC, TOPK, kFusedV, false>(ab, g, fp, red, linear, nk, nchunks, nprob);
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void approx_fused(ApproxBatch ab, Geometry g, FusedParams fp)
{
    __shared__ float red[4][kFusedJ * 64];
    const int linear = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    if (!BF16 && fp.rows3) { fused3_dispatch(ab, g, fp, red, linear, gridDim.x, gridDim.y, gridDim.z); return; }
    fused_dispatch<BF16, false, false>(ab, g, fp, red, linear, gridDim.x, gridDim.y, gridDim.z);
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void approx_fused_nhwc(ApproxBatch ab, Geometry g, FusedParams fp)
{
    __shared__ float red[4][kFusedJ * 64];
    const int linear = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    fused_dispatch<BF16, true, false>(ab, g, fp, red, linear, gridDim.x, gridDim.y, gridDim.z);
}

template <bool BF16>
__global__ __launch_bounds__(kBlock) void approx_fused_topk(ApproxBatch ab, Geometry g, FusedParams fp)
{
    __shared__ float red[4][kFusedJ * 64];
    const int linear = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    fused_dispatch<BF16, false, true>(ab, g, fp, red, linear, gridDim.x, gridDim.y, gridDim.z);
}

// Channel-last gather for the shapes the fused form does not take: one thread per VEC consecutive
// channels of one filter-gradient entry (k, r, s, c..) and batch chunk.  Consecutive lanes read
// consecutive channels of the same input pixel, the access pattern the paper's kernel is built on.
template <bool BF16, int VEC>
__global__ __launch_bounds__(kBlock) void nhwc_gather(const void *__restrict__ X, const int32_t *__restrict__ hw,
                                                      const float *__restrict__ sum, float *__restrict__ out,
                                                      Geometry g, int chunk_n, float scale, int dw_layout)
{
    const long o = ((long)blockIdx.x * kBlock + threadIdx.x) * VEC;     // (k, r, s, c) with c fastest
    const int RS = g.R * g.S, CRS = g.C * RS;
    if (o >= (long)g.K * CRS) return;
    const int k = (int)(o / CRS), j = (int)(o % CRS);
    const int tap = j / g.C, c = j % g.C, r = tap / g.S, s = tap % g.S;
    const int n_begin = blockIdx.y * chunk_n;
    const int n_end = n_begin + chunk_n < g.N ? n_begin + chunk_n : g.N;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
#pragma unroll 4
    for (int n = n_begin; n < n_end; ++n) {
        const int p = hw[(long)n * g.K + k];
        const float sv = sum[(long)n * g.K + k];
        const int ih = (p >> 16) * g.sh + r - g.ph, iw = (p & 0xffff) * g.sw + s - g.pw;
        if (ih >= 0 && ih < g.H && iw >= 0 && iw < g.W) {
            const long xi = (((long)n * g.H + ih) * g.W + iw) * g.C + c;
            float xv[VEC];
            if (VEC == 1) {
                xv[0] = BF16 ? bf16_bits_to_float(((const uint16_t *)X)[xi]) : ((const float *)X)[xi];
            } else if (BF16) {
                const uint2 raw = *(const uint2 *)((const uint16_t *)X + xi);
                xv[0] = __uint_as_float(raw.x << 16); xv[1] = __uint_as_float(raw.x & 0xffff0000u);
                xv[2] = __uint_as_float(raw.y << 16); xv[3] = __uint_as_float(raw.y & 0xffff0000u);
            } else {
                const float4 raw = *(const float4 *)((const float *)X + xi);
                xv[0] = raw.x; xv[1] = raw.y; xv[2] = raw.z; xv[3] = raw.w;
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[v] = fmaf(sv, xv[v], acc[v]);
        }
    }
    float *dst = out + (long)blockIdx.y * g.K * CRS;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        long at = o + v;
        if (dw_layout == WGRAD_DW_HWIO) at = (long)(j + v) * g.K + k;
        else if (dw_layout == WGRAD_DW_OIHW) at = ((long)k * g.C + c + v) * RS + tap;
        dst[at] = acc[v] * scale;
    }
}

// Several groups of layers (each group one geometry) in one launch: a workgroup looks its group up.
// The parameters are read through the kernel-argument segment pointer (indexing the by-value argument
// with a run-time group number would make the compiler copy all of it into scratch memory first).
constexpr int kFusedMultiMax = 6;
struct FusedGroup {
    ApproxBatch ab;
    Geometry g;
    FusedParams fp;
    int nchunks, nprob;
};
struct FusedMulti {
    int n;
    int begin[kFusedMultiMax + 1];   // first workgroup of each group, multiples of 8; begin[n] = grid size
    int count[kFusedMultiMax];
    FusedGroup grp[kFusedMultiMax];
};

template <bool BF16, bool TOPK = false>
__global__ __launch_bounds__(kBlock) void approx_fused_multi(const FusedMulti)
{
    __shared__ float red[4][kFusedJ * 64];
    const FusedMulti *mp = (const FusedMulti *)__builtin_amdgcn_kernarg_segment_ptr();
    const int n = mp->n;
    int gi = 0;
    for (int i = 1; i < n; ++i) gi += (int)blockIdx.x >= mp->begin[i];
    const int linear = (int)blockIdx.x - mp->begin[gi];
    if (linear >= mp->count[gi]) return;
    FTRACE_G(gi);
    const FusedGroup &G = mp->grp[gi];
    if (!BF16 && !TOPK && G.fp.rows3) fused3_dispatch(G.ab, G.g, G.fp, red, linear, G.g.K * G.fp.nslice, G.nchunks, G.nprob);
    else fused_dispatch<BF16, false, TOPK>(G.ab, G.g, G.fp, red, linear, G.g.K * G.fp.nslice, G.nchunks, G.nprob);
    FTRACE(3);
}

WGRAD_FUSED_TRACE_READER(wgrad_debug_read_trace_fused)

struct FusedQueue {
    int n = 0, bf16 = 0, topk = 0;   // groups of one element type and one form (k = 1 or top-k) per launch
    FusedGroup grp[kFusedMultiMax];
};

int fused_flush(FusedQueue &q, hipStream_t st)
{
    if (q.n == 0) return WGRAD_OK;
    FusedMulti m{};
    m.n = q.n;
    long blocks = 0;
    for (int i = 0; i < q.n; ++i) {
        m.grp[i] = q.grp[i];
        m.begin[i] = (int)blocks;
        m.count[i] = q.grp[i].g.K * q.grp[i].fp.nslice * q.grp[i].nchunks * q.grp[i].nprob;
        blocks += (m.count[i] + 7) / 8 * 8;
    }
    m.begin[q.n] = (int)blocks;
    const bool bf16 = q.bf16, topk = q.topk;
    q.n = 0;
    if (blocks >= (1l << 31)) return WGRAD_UNSUPPORTED;
#define FM_ARGS dim3((unsigned)blocks), dim3(kBlock), 0, st, m
    if (topk) { if (bf16) WGRAD_LAUNCH((approx_fused_multi<true, true>), FM_ARGS); else WGRAD_LAUNCH((approx_fused_multi<false, true>), FM_ARGS); }
    else      { if (bf16) WGRAD_LAUNCH((approx_fused_multi<true, false>), FM_ARGS); else WGRAD_LAUNCH((approx_fused_multi<false, false>), FM_ARGS); }
#undef FM_ARGS
    return launch_status();
}

#ifndef WGRAD_APPROX_THREADS   // threads to aim for when chunking the batch (direct form)
#define WGRAD_APPROX_THREADS (256 * 1024)
#endif
#ifndef WGRAD_GATHER_BLOCKS    // workgroups to aim for (LDS form)
#define WGRAD_GATHER_BLOCKS 512
#endif

ApproxPlan plan_approx(const Geometry &g, bool allow_lds, bool allow_fused, bool allow_mm)
{
    ApproxPlan pl{};
    const long outs = g.dw_elems();
    const int HW = g.H * g.W;
    // bf16 inputs, shapes the bf16 matrix-core kernel takes: the approximated gradient is the exact
    // one of the sparsified dY (Section 2.4), and contracting that on the matrix core -- the operand
    // built in registers from each map's selected position and sum -- outruns any gather from LDS
    // (16 K multiply-adds per instruction against 64), even though all but one of a map's slots are zero
    // -- up to maps of 256 positions; beyond, the fused kernel below is bound by its dY stream and wins
    if (allow_mm && g.bf16 && g.Ho * g.Wo <= 256 && tune_int("WGRAD_APPROX_MM", 1)) {
        const ExactPlan ex = plan_exact(g);
        if (ex.ok && ex.mm16) {
            pl.mm = 1;
            pl.ex = ex;
            pl.chunks = ex.splits; pl.chunk_n = 0;
            size_t off = 0;
            pl.off_idx = off; off += align_up((size_t)g.N * g.K * 4);
            pl.off_sum = off; off += align_up((size_t)g.N * g.K * 4);
            pl.off_part = off; off += ex.splits > 1 ? align_up((size_t)ex.splits * outs * 4) : 0;
            pl.ws_bytes = off;
            const size_t alt = plan_approx(g, false, false, false).ws_bytes;
            if (alt > pl.ws_bytes) pl.ws_bytes = alt;
            return pl;
        }
    }
    // fp32 inputs on planes of up to four positions: the exact matrix-core kernel on the sparsified dY
    if (allow_mm && !g.bf16 && g.Ho * g.Wo <= 4 && tune_int("WGRAD_APPROX_SX", 1)) {
        const ExactPlan ex = plan_exact(g);
        if (ex.ok && ex.stream) {
            pl.sx = 1;
            pl.ex = ex;
            pl.chunks = 1; pl.chunk_n = g.N;
            pl.off_sparse = 0;
            pl.off_part = align_up((size_t)g.N * g.K * g.Ho * g.Wo * 4);
            pl.ws_bytes = pl.off_part + align_up(ex.ws_bytes);
            return pl;
        }
    }
    // LDS form when every input element is used several times over by the K patches of its image
    // haloed plane: rows/cols -pad .. max(last tap the positions can reach, last row/col of X)
    const int hp = std::max((g.Ho - 1) * g.sh + 3, g.H + g.ph), wp = std::max((g.Wo - 1) * g.sw + 3, g.W + g.pw);
    const int pitch = (hp * wp) | 1;
    pl.use_lds = allow_lds && g.R == 3 && g.S == 3 && g.C >= 16 && g.K >= 128 && (long)g.K * 9 >= 2l * HW && HW % 4 == 0
                 && kGatherCT * HW <= kGatherSlots * kGatherBlock * 4
                 && (size_t)2 * kGatherCT * pitch * 4 <= kGatherLds;
    long chunks;
    if (pl.use_lds) {
        // output channels per wavefront: four where K allows (the work between two barriers doubles against two, the
        // re-staging of X per output channel halves: VGG-19 fp32 approximation phase -6 %)
        pl.m = g.K >= 256 ? 4 : 1;
        pl.pitch = pitch;
        pl.wp = wp;
        // images per group: at most 8 16-byte loads per thread, one lane per (image, channel) pair
        pl.nb = kGatherSlots * kGatherBlock * 4 / (kGatherCT * HW);
        if (pl.nb > 64 / pl.m) pl.nb = 64 / pl.m;
        const int lds_cap = (int)(kGatherLds / ((size_t)2 * kGatherCT * pl.pitch * 4));   // double buffered
        if (pl.nb > lds_cap) pl.nb = lds_cap;
        if (pl.nb > g.N) pl.nb = g.N;
        pl.ctiles = (g.C + kGatherCT - 1) / kGatherCT;
        pl.ktiles = (g.K + 8 * pl.m - 1) / (8 * pl.m);
        const long tiles = (long)pl.ctiles * pl.ktiles;
        const int want_blocks = tune_int("WGRAD_GATHER_BLOCKS", WGRAD_GATHER_BLOCKS);
        chunks = tiles >= want_blocks ? 1 : (want_blocks + tiles - 1) / tiles;
        const long max_chunks = (g.N + pl.nb - 1) / pl.nb;
        if (chunks > max_chunks) chunks = max_chunks;
        // the batch-chunk partial sums are written and read once each: never more than 20 MiB of them
        const long by_bytes = (20l << 20) / (outs * 4) < 1 ? 1 : (20l << 20) / (outs * 4);
        if (chunks > by_bytes) chunks = by_bytes;
    } else if (allow_fused && tune_int("WGRAD_APPROX_FUSED", 1) && (g.Ho * g.Wo) % 4 == 0
               && g.Ho * g.Wo <= 64 * kFusedV * 4 && g.crs() <= 64 * kFusedJ * kFusedSlices && g.R * g.S <= 63
               && ((long)g.H + 2l * g.ph + g.R) * ((long)g.W + 2l * g.pw + g.S) * g.C < (1l << 24)) {
        // (the last two: a tap's number and its offset inside the padded input share one 32-bit word)
        // fused form: one workgroup per (output channel, batch chunk); four images at a time
        pl.fused = 1;
        const long wgs = (long)g.K * fused_slices(g);
        chunks = (tune_int("WGRAD_FUSED_BLOCKS", 768) + wgs - 1) / wgs;
        if (chunks > (g.N + 7) / 8) chunks = (g.N + 7) / 8;         // at least two images per wavefront
    } else {
        chunks = (tune_int("WGRAD_APPROX_THREADS", WGRAD_APPROX_THREADS) + outs - 1) / outs;
        if (chunks > g.N) chunks = g.N;
    }
    if (chunks < 1) chunks = 1;
    pl.chunk_n = (int)((g.N + chunks - 1) / chunks);
    pl.chunks = (g.N + pl.chunk_n - 1) / pl.chunk_n;
    size_t off = 0;
    pl.off_idx = off; off += align_up((size_t)g.N * g.K * 4);
    pl.off_sum = off; off += align_up((size_t)g.N * g.K * 4);
    pl.off_part = off; off += pl.chunks > 1 ? align_up((size_t)pl.chunks * outs * 4) : 0;
    pl.ws_bytes = off;
    // tensors that are not 16-byte aligned get the three-kernel direct form: size the workspace for both
    if (pl.use_lds || pl.fused) {
        const size_t alt = plan_approx(g, false, false).ws_bytes;
        if (alt > pl.ws_bytes) pl.ws_bytes = alt;
    }
    return pl;
}

static GatherParams gather_params(const ApproxPlan &pl, const Geometry &g, float scale)
{
    GatherParams gp;
    gp.ctiles = pl.ctiles; gp.nb = pl.nb; gp.chunk_n = pl.chunk_n; gp.wp = pl.wp; gp.pitch = pl.pitch;
    gp.d_hw4 = FastDiv(g.H * g.W / 4);        // dividends stay below 64 * H*W, far under the 2^32 bound
    gp.d_w = FastDiv(g.W);
    gp.scale = scale;
    gp.tk = 1; gp.inv_k = 1.0f;
    return gp;
}

template <bool BF16>
static void launch_gather_lds(const ApproxPlan &pl, dim3 grid, size_t lds, hipStream_t st, const ApproxBatch &ab,
                              const Geometry &g, float scale)
{
    const GatherParams gp = gather_params(pl, g, scale);
#define GL_ARGS grid, dim3(kGatherBlock), lds, st, ab, g, gp
    if (pl.m == 4) WGRAD_LAUNCH((approx_gather_lds3x3<BF16, 4>), GL_ARGS);
    else WGRAD_LAUNCH((approx_gather_lds3x3<BF16, 1>), GL_ARGS);
#undef GL_ARGS
}

// LDS gathers of a schedule run collected for one launch: groups of one element type and one M
struct GatherQueue {
    SelectQueue *sel = nullptr;      // selections that must be issued before these gathers
    int n = 0, bf16 = 0, m = 0;
    size_t lds = 0;                  // the largest window buffer among the groups
    int nprob[kGatherMultiMax];
    GatherGroup grp[kGatherMultiMax];
};

GatherQueue *gather_queue_new(SelectQueue *selects)
{
    GatherQueue *q = new GatherQueue;
    q->sel = selects;
    return q;
}
void gather_queue_delete(GatherQueue *q) { delete q; }

int gather_flush(GatherQueue &q, hipStream_t st)
{
    if (q.n == 0) return WGRAD_OK;
    if (q.sel) {
        const int rc = select_flush(*q.sel, st);
        if (rc != WGRAD_OK) return rc;
    }
    GatherMulti m{};
    m.n = q.n;
    long blocks = 0;
    for (int i = 0; i < q.n; ++i) {
        m.grp[i] = q.grp[i];
        m.begin[i] = (int)blocks;
        blocks += (long)q.grp[i].gx * q.grp[i].gy * q.nprob[i];
    }
    m.begin[q.n] = (int)blocks;
    const int bf16 = q.bf16, mm = q.m;
    const size_t lds = q.lds;
    q.n = 0; q.lds = 0;
    if (blocks >= (1l << 31)) return WGRAD_UNSUPPORTED;
#define GM_ARGS dim3((unsigned)blocks), dim3(kGatherBlock), lds, st, m
    if (bf16) { if (mm == 4) WGRAD_LAUNCH((approx_gather_lds_multi<true, 4>), GM_ARGS); else WGRAD_LAUNCH((approx_gather_lds_multi<true, 1>), GM_ARGS); }
    else      { if (mm == 4) WGRAD_LAUNCH((approx_gather_lds_multi<false, 4>), GM_ARGS); else WGRAD_LAUNCH((approx_gather_lds_multi<false, 1>), GM_ARGS); }
#undef GM_ARGS
    return launch_status();
}

// Batch-chunk partials (bytes) that the top-k forms borrowed from this file may need.
size_t topk_borrowed_partial_bytes(const Geometry &g)
{
    size_t need = 0;
    const ApproxPlan a = plan_approx(g, true, false, false), b = plan_approx(g, false, true, false);
    if (a.use_lds && a.chunks > 1) need = (size_t)a.chunks * g.dw_elems() * 4;
    if (b.fused && b.chunks > 1 && (size_t)b.chunks * g.dw_elems() * 4 > need) need = (size_t)b.chunks * g.dw_elems() * 4;
    return need;
}

// Whether the top-k form of this shape is the fused kernel's: its shape class, unless the LDS gather takes the
// shape (many output channels on small planes), which is the faster of the two there.
bool topk_takes_fused(const Geometry &g, int k)
{
    const ApproxPlan lds = plan_approx(g, /*allow_lds=*/true, /*allow_fused=*/false, /*allow_mm=*/false);
    if (lds.use_lds && lds.m * k <= 64) return false;
    return plan_approx(g, /*allow_lds=*/false, /*allow_fused=*/true, /*allow_mm=*/false).fused != 0;
}

// Top-k through the fused kernel (selection and gather in one launch, positions never leave registers).
// False if the shape is not one the fused form takes.
// b: one problem, or (schedule runs) several layers of this geometry; problem i keeps its batch-chunk partials at
// partials + i * partial_stride floats.
bool topk_fused(const Geometry &g, const Batch &b, int k, float scale,
                int32_t *idx_out, float *sum_out, float *partials, long partial_stride, hipStream_t st, int *rc,
                FusedQueue *fq, CombineQueue *defer)
{
    if (!topk_takes_fused(g, k)) return false;
    ApproxPlan pl = plan_approx(g, /*allow_lds=*/false, /*allow_fused=*/true, /*allow_mm=*/false);
    if (!pl.fused) return false;
    for (int i = 0; i < b.n; ++i)
        if (((uintptr_t)b.dY[i] % (g.bf16 ? 8 : 16)) != 0) return false;
    if (!defer || idx_out || sum_out) fq = nullptr;    // a queued launch needs its reduction queued behind it
    if (fq) {
        // part of a launch of many layers: chunk for eight images per wavefront (see launch_approx), never finer
        // than planned (the workspace holds pl.chunks partials)
        const int chunks = (g.N + 4 * 8 - 1) / (4 * 8);
        if (chunks >= 1 && chunks < pl.chunks) {
            pl.chunk_n = (g.N + chunks - 1) / chunks;
            pl.chunks = (g.N + pl.chunk_n - 1) / pl.chunk_n;
        }
    }
    const long outs = g.dw_elems();
    ApproxBatch ab{};
    for (int i = 0; i < kMaxBatch; ++i) {
        const int j = i < b.n ? i : 0;
        ab.X[i] = b.X[j]; ab.dY[i] = b.dY[j];
        ab.out[i] = pl.chunks > 1 ? partials + j * partial_stride : b.dW[j];
    }
    FusedParams fp;
    fp.chunk_n = pl.chunk_n; fp.scale = pl.chunks > 1 ? 1.0f : scale;
    fp.d_rs = FastDiv(g.R * g.S); fp.d_s = FastDiv(g.S); fp.d_wo = FastDiv(g.Wo);
    fp.flat_out = idx_out; fp.sum_out = sum_out; fp.dw_layout = WGRAD_DW_OIHW; fp.tk = k; fp.inv_k = 1.0f / k; fp.nslice = fused_slices(g); fp.slice_major = tune_int("WGRAD_FUSED_SLICE_MAJOR", 1);
    fp.rows3 = 0; fp.d_r = FastDiv(g.R);
    if (fq) {
        if (fq->n == kFusedMultiMax || (fq->n > 0 && (fq->bf16 != g.bf16 || !fq->topk))) {
            *rc = fused_flush(*fq, st);
            if (*rc != WGRAD_OK) return true;
        }
        FusedGroup &G = fq->grp[fq->n++];
        fq->bf16 = g.bf16; fq->topk = 1;
        G.ab = ab; G.g = g; G.fp = fp; G.nchunks = pl.chunks; G.nprob = b.n;
        *rc = WGRAD_OK;
    } else {
        const dim3 grid(g.K * fp.nslice, pl.chunks, (unsigned)b.n);
        if (g.bf16) WGRAD_LAUNCH((approx_fused_topk<true>), grid, dim3(kBlock), 0, st, ab, g, fp);
        else        WGRAD_LAUNCH((approx_fused_topk<false>), grid, dim3(kBlock), 0, st, ab, g, fp);
        *rc = launch_status();
    }
    if (*rc == WGRAD_OK && pl.chunks > 1)
        *rc = launch_combine(partials, partial_stride, pl.chunks, outs, scale, b.dW, b.n, st, fq ? defer : nullptr);
    return true;
}

// The LDS gather over the kept positions of the top-k form.  False if the shape is not one the LDS
// form takes (the caller then uses its general gather); rc receives the launch status otherwise.
bool topk_gather_lds(const Geometry &g, const void *X, const int32_t *hw, const float *sum, int k, float scale,
                     float *dW, float *partials, size_t partial_cap_bytes, hipStream_t st, int *rc)
{
    ApproxPlan pl = plan_approx(g, /*allow_lds=*/true, /*allow_fused=*/false, /*allow_mm=*/false);
    if (!pl.use_lds || pl.m * k > 64 || ((uintptr_t)X % (g.bf16 ? 8 : 16)) != 0) return false;
    if (pl.nb > 64 / (pl.m * k)) pl.nb = 64 / (pl.m * k);
    const long outs = g.dw_elems();
    if (pl.chunks > 1 && (size_t)pl.chunks * outs * 4 > partial_cap_bytes) return false;
    ApproxBatch ab{};
    for (int i = 0; i < kMaxBatch; ++i) {
        ab.X[i] = X; ab.hw[i] = const_cast<int32_t *>(hw); ab.sum[i] = const_cast<float *>(sum);
        ab.out[i] = pl.chunks > 1 ? partials : dW;
    }
    GatherParams gp;
    gp.ctiles = pl.ctiles; gp.nb = pl.nb; gp.chunk_n = pl.chunk_n; gp.wp = pl.wp; gp.pitch = pl.pitch;
    gp.d_hw4 = FastDiv(g.H * g.W / 4);
    gp.d_w = FastDiv(g.W);
    gp.scale = pl.chunks > 1 ? 1.0f : scale;
    gp.tk = k; gp.inv_k = 1.0f / k;
    const dim3 grid(pl.ctiles * pl.ktiles, pl.chunks, 1);
    const size_t lds = (size_t)2 * pl.nb * kGatherCT * pl.pitch * 4;
#define GL_ARGS grid, dim3(kGatherBlock), lds, st, ab, g, gp
    if (g.bf16) { if (pl.m == 4) WGRAD_LAUNCH((approx_gather_lds3x3<true, 4, true>), GL_ARGS);
                  else           WGRAD_LAUNCH((approx_gather_lds3x3<true, 1, true>), GL_ARGS); }
    else        { if (pl.m == 4) WGRAD_LAUNCH((approx_gather_lds3x3<false, 4, true>), GL_ARGS);
                  else           WGRAD_LAUNCH((approx_gather_lds3x3<false, 1, true>), GL_ARGS); }
#undef GL_ARGS
    *rc = launch_status();
    if (*rc == WGRAD_OK && pl.chunks > 1) {
        float *dst[1] = {dW};
        *rc = launch_combine(partials, 0, pl.chunks, outs, scale, dst, 1, st, nullptr);
    }
    return true;
}

int launch_approx(const Geometry &g, const ApproxPlan &plan, const Batch &b, float scale,
                  int32_t *idx_out, float *sum_out, void *ws, hipStream_t st, CombineQueue *defer, FusedQueue *fq,
                  Bf16Queue *bq, GatherQueue *gq, SelectQueue *sq)
{
    // a queued launch needs its reduction queued behind it: without a reduction queue nothing is queued
    if (!defer) { gq = nullptr; fq = nullptr; bq = nullptr; sq = nullptr; }
    bool aligned = true;
    for (int i = 0; i < b.n; ++i)
        aligned = aligned && ((uintptr_t)b.X[i] % (g.bf16 ? 8 : 16)) == 0 && ((uintptr_t)b.dY[i] % (g.bf16 ? 8 : 16)) == 0;
    ApproxPlan pl = ((plan.use_lds || plan.fused || plan.mm) && !aligned) ? plan_approx(g, false, false, false) : plan;   // (the sparsified form has no alignment needs: the exact launcher falls back by itself)
    const long outs = g.dw_elems();
    if (pl.use_lds && (b.n > 1 || gq)) {
        // the workgroup target is for the whole launch: a batch of layers chunks each layer's images less finely
        const long tiles = (long)pl.ctiles * pl.ktiles * b.n;
        // (a group that shares its launch with others: half as many, longer workgroups -- the next group's fill the chip
        // as these finish, and the partial sums halve)
        const int want_blocks = gq ? tune_int("WGRAD_GATHER_BLOCKS_SHARED", WGRAD_GATHER_BLOCKS / 2)
                                   : tune_int("WGRAD_GATHER_BLOCKS", WGRAD_GATHER_BLOCKS);
        long chunks = tiles >= want_blocks ? 1 : (want_blocks + tiles - 1) / tiles;
        if (chunks < pl.chunks) {       // never more than planned: the workspace holds pl.chunks partials
            pl.chunk_n = (int)((g.N + chunks - 1) / chunks);
            pl.chunks = (g.N + pl.chunk_n - 1) / pl.chunk_n;
        }
    }
    if (pl.fused && (b.n > 1 || fq)) {
        long chunks;
        if (fq) {
            // part of a launch of many groups, which fills the chip anyway: chunk for the images a wavefront
            // walks -- eight: fewer (more, shorter workgroups) loses to the per-workgroup set-up and to the
            // larger partial sums, more leaves too few workgroups to balance the tail
            const int per_wave = tune_int("WGRAD_FUSED_IPW", 8);
            chunks = (g.N + 4 * per_wave - 1) / (4 * per_wave);
        } else {
            // the workgroup target is for the whole launch: a batch chunks each problem less finely
            const long wgs = (long)g.K * fused_slices(g) * b.n;
            chunks = (tune_int("WGRAD_FUSED_BLOCKS", 768) + wgs - 1) / wgs;
        }
        if (chunks < 1) chunks = 1;
        if (chunks < pl.chunks) {       // never more than planned: the workspace holds pl.chunks partials
            pl.chunk_n = (int)((g.N + chunks - 1) / chunks);
            pl.chunks = (g.N + pl.chunk_n - 1) / pl.chunk_n;
        }
    }
    // problem i owns the i-th slice (plan.ws_bytes each) of the workspace
    ApproxBatch ab{};
    for (int i = 0; i < kMaxBatch; ++i) {
        const int j = i < b.n ? i : 0;
        char *slice = (char *)ws + (size_t)j * plan.ws_bytes;
        ab.X[i] = b.X[j]; ab.dY[i] = b.dY[j];
        ab.hw[i] = (int32_t *)(slice + pl.off_idx);
        ab.sum[i] = (float *)(slice + pl.off_sum);
        ab.out[i] = pl.chunks > 1 ? (float *)(slice + pl.off_part) : b.dW[j];
    }
    const float kscale = pl.chunks > 1 ? 1.0f : scale;
    int rc;
    if (pl.sx) {
        // the group's workspace (b.n slices of plan.ws_bytes, contiguous) is cut anew: the sparsified tensors of
        // all problems first, then one region for the exact kernel's partials of the whole batch
        ApproxBatch sb{};
        Batch eb{};
        eb.n = b.n;
        for (int i = 0; i < kMaxBatch; ++i) {
            const int j = i < b.n ? i : 0;
            sb.dY[i] = b.dY[j];
            sb.out[i] = (float *)((char *)ws + (size_t)j * pl.off_part);
            eb.X[i] = b.X[j]; eb.dY[i] = sb.out[i]; eb.dW[i] = b.dW[j];
        }
        const long maps = (long)g.N * g.K;
        const dim3 grid((unsigned)((maps + kBlock - 1) / kBlock), (unsigned)b.n);
        WGRAD_LAUNCH(sparsify_small, grid, dim3(kBlock), 0, st, sb, maps, g.Ho * g.Wo, scale, idx_out, sum_out);
        rc = launch_status();
        if (rc != WGRAD_OK) return rc;
        return launch_exact(g, pl.ex, eb, (char *)ws + (size_t)b.n * pl.off_part, st, defer);
    }
    bool aligned16 = true;
    for (int i = 0; i < b.n; ++i) aligned16 = aligned16 && ((uintptr_t)b.X[i] % 16) == 0;
    if (pl.mm && planes_bf16_takes(g) && aligned16 && (!bq || g.H <= tune_int("WGRAD_BF16_PLANES_APPROX_SHARED_HW", 2))) {
        // 2x2 planes, and 4x4 planes in single calls: the position-major kernel, its A operand built from the
        // selections; it writes dW itself.  (In a schedule run the selections and the sparse-operand launches of the
        // layers on 4x4 planes share launches with the other layers', which measured faster than this kernel with a
        // selection and a launch per group.)
        rc = launch_select_impl(g, ab, b.n, idx_out, sum_out, st, nullptr);
        if (rc != WGRAD_OK) return rc;
        SparseA sp{};
        for (int i = 0; i < b.n; ++i) { sp.hw[i] = ab.hw[i]; sp.sum[i] = ab.sum[i]; }
        sp.scale = scale;
        return launch_exact_bf16_planes(g, b, st, &sp);
    }
    if (pl.mm) {
        rc = launch_select_impl(g, ab, b.n, idx_out, sum_out, st, bq ? sq : nullptr);   // (a queued consumer issues queued selections first)
        if (rc != WGRAD_OK) return rc;
        ExactPlan ex = pl.ex;
        if (b.n > 1) {
            const int splits = choose_splits(ex, b.n);
            if (splits < ex.splits) ex.splits = splits;
        }
        if (bq) {
            // one of several groups in a launch: fewer, longer workgroups (see launch_exact); the sparse operand
            // costs no loads, so the partial results weigh more here and the best count is lower still
            const int splits = choose_splits(ex, b.n, tune_int("WGRAD_BF16_MULTI_BLOCKS_SPARSE", 128));
            if (splits < ex.splits) ex.splits = splits;
        }
        SparseA sp{};
        float *out[kMaxBatch];
        const long prob_stride = (long)(plan.ws_bytes / 4);
        for (int i = 0; i < b.n; ++i) {
            sp.hw[i] = ab.hw[i]; sp.sum[i] = ab.sum[i];
            out[i] = ex.splits > 1 ? (float *)((char *)ws + (size_t)i * plan.ws_bytes + pl.off_part) : b.dW[i];
        }
        sp.scale = ex.splits > 1 ? 1.0f : scale;
        rc = launch_exact_bf16(g, ex, b, out, st, &sp, bq);
        if (rc != WGRAD_OK) return rc;
        if (ex.splits > 1)
            return launch_combine((const float *)((char *)ws + pl.off_part), prob_stride, ex.splits, outs, scale, b.dW, b.n, st, defer);
        return WGRAD_OK;
    }
    if (pl.fused) {
        FusedParams fp;
        fp.chunk_n = pl.chunk_n; fp.scale = kscale;
        fp.d_rs = FastDiv(g.R * g.S); fp.d_s = FastDiv(g.S); fp.d_wo = FastDiv(g.Wo);
        fp.flat_out = idx_out; fp.sum_out = sum_out; fp.dw_layout = WGRAD_DW_OIHW; fp.tk = 1; fp.inv_k = 1.0f; fp.nslice = fused_slices(g); fp.slice_major = tune_int("WGRAD_FUSED_SLICE_MAJOR", 1);
        fp.rows3 = tune_int("WGRAD_FUSED_ROWS3", 1) ? fused_rows3(g) : 0; fp.d_r = FastDiv(g.R);
        if (fq) {
            // part of a multi-group launch (groups of one element type)
            if (fq->n == kFusedMultiMax || (fq->n > 0 && (fq->bf16 != g.bf16 || fq->topk))) {
                rc = fused_flush(*fq, st);
                if (rc != WGRAD_OK) return rc;
            }
            FusedGroup &G = fq->grp[fq->n++];
            fq->bf16 = g.bf16; fq->topk = 0;
            G.ab = ab; G.g = g; G.fp = fp; G.nchunks = pl.chunks; G.nprob = b.n;
        } else {
            const dim3 grid((unsigned)(g.K * fp.nslice), (unsigned)pl.chunks, (unsigned)b.n);
            if (g.bf16) WGRAD_LAUNCH((approx_fused<true>), grid, dim3(kBlock), 0, st, ab, g, fp);
            else        WGRAD_LAUNCH((approx_fused<false>), grid, dim3(kBlock), 0, st, ab, g, fp);
            rc = launch_status();
            if (rc != WGRAD_OK) return rc;
        }
        if (pl.chunks > 1)
            return launch_combine((const float *)((char *)ws + pl.off_part), (long)(plan.ws_bytes / 4), pl.chunks, outs,
                                  scale, b.dW, b.n, st, defer);
        return WGRAD_OK;
    }
    rc = launch_select_impl(g, ab, b.n, idx_out, sum_out, st, pl.use_lds && gq ? sq : nullptr);
    if (rc != WGRAD_OK) return rc;

    if (pl.use_lds && gq) {
        // part of a multi-group launch (groups of one element type and one M); its reduction is deferred with the others
        if (gq->n == kGatherMultiMax || (gq->n > 0 && (gq->bf16 != g.bf16 || gq->m != pl.m))) {
            rc = gather_flush(*gq, st);
            if (rc != WGRAD_OK) return rc;
        }
        const size_t lds = (size_t)2 * pl.nb * kGatherCT * pl.pitch * 4;
        GatherGroup &G = gq->grp[gq->n];
        gq->nprob[gq->n++] = b.n;
        gq->bf16 = g.bf16; gq->m = pl.m;
        if (lds > gq->lds) gq->lds = lds;
        G.ab = ab; G.g = g; G.gp = gather_params(pl, g, kscale); G.gx = pl.ctiles * pl.ktiles; G.gy = pl.chunks;
        if (pl.chunks > 1)
            return launch_combine((const float *)((char *)ws + pl.off_part), (long)(plan.ws_bytes / 4), pl.chunks, outs,
                                  scale, b.dW, b.n, st, defer);
        return WGRAD_OK;
    }
    if (pl.use_lds) {
        const dim3 grid((unsigned)(pl.ctiles * pl.ktiles), (unsigned)pl.chunks, (unsigned)b.n);
        const size_t lds = (size_t)2 * pl.nb * kGatherCT * pl.pitch * 4;
        if (g.bf16) launch_gather_lds<true>(pl, grid, lds, st, ab, g, kscale);
        else        launch_gather_lds<false>(pl, grid, lds, st, ab, g, kscale);
    } else {
        const dim3 grid((unsigned)((outs + kBlock - 1) / kBlock), (unsigned)pl.chunks, (unsigned)b.n);
        if (g.bf16) WGRAD_LAUNCH((approx_gather_direct<true>), grid, dim3(kBlock), 0, st, ab, g, pl.chunk_n, kscale);
        else        WGRAD_LAUNCH((approx_gather_direct<false>), grid, dim3(kBlock), 0, st, ab, g, pl.chunk_n, kscale);
    }
    rc = launch_status();
    if (rc != WGRAD_OK) return rc;
    if (pl.chunks > 1)
        return launch_combine((const float *)((char *)ws + pl.off_part), (long)(plan.ws_bytes / 4), pl.chunks, outs,
                              scale, b.dW, b.n, st, defer);
    return WGRAD_OK;
}

FusedQueue *fused_queue_new() { return new FusedQueue; }
void fused_queue_delete(FusedQueue *q) { delete q; }

// ---- channel-last input (Section 2.4: the layouts of the paper's kernel) ----
static ApproxPlan plan_approx_nhwc(const Geometry &g)
{
    return plan_approx(g, /*allow_lds=*/false, /*allow_fused=*/true, /*allow_mm=*/false);
}

size_t approx_nhwc_ws_bytes(const Geometry &g) { return plan_approx_nhwc(g).ws_bytes; }

int launch_approx_nhwc(const Geometry &g, const void *X, const void *dY, float *dW, int dw_layout, float scale,
                       int32_t *idx_out, float *sum_out, void *ws, hipStream_t st)
{
    ApproxPlan pl = plan_approx_nhwc(g);
    if (pl.fused && ((uintptr_t)dY % (g.bf16 ? 8 : 16)) != 0) pl = plan_approx(g, false, false, false);
    const long outs = g.dw_elems();
    ApproxBatch ab{};
    for (int i = 0; i < kMaxBatch; ++i) {
        ab.X[i] = X; ab.dY[i] = dY;
        ab.hw[i] = (int32_t *)((char *)ws + pl.off_idx);
        ab.sum[i] = (float *)((char *)ws + pl.off_sum);
        ab.out[i] = pl.chunks > 1 ? (float *)((char *)ws + pl.off_part) : dW;
    }
    const float kscale = pl.chunks > 1 ? 1.0f : scale;
    int rc;
    if (pl.fused) {
        FusedParams fp;
        fp.chunk_n = pl.chunk_n; fp.scale = kscale;
        fp.d_rs = FastDiv(g.C); fp.d_s = FastDiv(g.S); fp.d_wo = FastDiv(g.Wo);
        fp.flat_out = idx_out; fp.sum_out = sum_out; fp.dw_layout = dw_layout; fp.tk = 1; fp.inv_k = 1.0f; fp.nslice = fused_slices(g); fp.slice_major = tune_int("WGRAD_FUSED_SLICE_MAJOR", 1);
        fp.rows3 = 0; fp.d_r = FastDiv(g.R);
        const dim3 grid(g.K * fp.nslice, pl.chunks, 1);
        if (g.bf16) WGRAD_LAUNCH((approx_fused_nhwc<true>), grid, dim3(kBlock), 0, st, ab, g, fp);
        else        WGRAD_LAUNCH((approx_fused_nhwc<false>), grid, dim3(kBlock), 0, st, ab, g, fp);
        rc = launch_status();
    } else {
        rc = launch_select_impl(g, ab, 1, idx_out, sum_out, st);
        if (rc != WGRAD_OK) return rc;
        const bool vec = g.C % 4 == 0 && ((uintptr_t)X % (g.bf16 ? 8 : 16)) == 0;
        const long threads = vec ? outs / 4 : outs;
        const dim3 grid((unsigned)((threads + kBlock - 1) / kBlock), pl.chunks);
#define NG_ARGS grid, dim3(kBlock), 0, st, X, ab.hw[0], ab.sum[0], ab.out[0], g, pl.chunk_n, kscale, dw_layout
        if (g.bf16) { if (vec) WGRAD_LAUNCH((nhwc_gather<true, 4>), NG_ARGS); else WGRAD_LAUNCH((nhwc_gather<true, 1>), NG_ARGS); }
        else        { if (vec) WGRAD_LAUNCH((nhwc_gather<false, 4>), NG_ARGS); else WGRAD_LAUNCH((nhwc_gather<false, 1>), NG_ARGS); }
#undef NG_ARGS
        rc = launch_status();
    }
    if (rc != WGRAD_OK || pl.chunks == 1) return rc;
    float *dst[1] = {dW};
    return launch_combine((const float *)((char *)ws + pl.off_part), 0, pl.chunks, outs, scale, dst, 1, st, nullptr);
}

}  // namespace wgrad
