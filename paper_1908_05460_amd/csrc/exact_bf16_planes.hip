// Exact filter gradient for bf16 inputs on 2x2 and 4x4 planes (3x3 filters, stride 1, padding 1), position-major:
//
//     dW[k][c][r][s] = sum over positions p = (h, w) whose tap (r, s) lies inside X, q = (h + r - 1, w + s - 1), of
//                      G_pq[k][c],     G_pq[k][c] = sum_n dY[n][k][p] * X[n][c][q]                      (Section 2.4)
//
// Every G_pq is a plain matrix product whose only reduction dimension is the batch, so the operands of
// v_mfma_f32_16x16x32_bf16 are "32 images of one position": no window, no halo, and the (position, tap) pairs whose
// tap falls into the padding are never multiplied at all -- 16 of 36 pairs remain on a 2x2 plane, 100 of 144 on a
// 4x4 plane, which the row-window kernel (exact_bf16_kernel.hpp) multiplies with zeros.
//
// The tensors are position-minor in memory (a plane of a (n, k) map is contiguous), the operands want the batch
// minor: a stage of 32 images is transposed on its way into LDS.  A thread loads the same 8 positions (4 on a 2x2
// plane) of one channel for 8 consecutive images, transposes the 8x8 block of bf16 in registers (one byte-permute
// per output word) and writes one 16-byte piece per position: LDS holds [position][channel][32 images], the 16-byte
// pieces of a row XOR-swizzled with bits of the channel so that the 16 rows of an operand read spread over all banks.
// A workgroup owns 32 output channels x 64 (2x2) or 32 (4x4) input channels and walks the whole batch; its four
// wavefronts are 2 x 2 tiles of 16 output channels x 32 or 16 input channels.  No split of the reduction, no partial
// sums.  LDS is double-buffered and so are the staging registers: while four wavefronts multiply stage t, four others
// transpose stage t + 1 into the other buffer and have the loads of stage t + 2 in flight.
// What bounds it: the operands are read out of LDS twice (two wavefronts share each 16-row tile), about one LDS
// byte-cycle per matrix cycle, and every operand row is fetched once per tile column (row) of the result, K / 32 or
// C / 32 times, out of the L2 -- 512 -> 512 @ 4x4, N = 512: 37 us against 60 for the row-window kernel, 12 at the
// matrix core's rate.  Tiles of 64 x 64 on the 32x32x16 instruction (half the LDS bytes per product, half the
// fetches) were built and measured no faster: a layer then has 64 tiles for 256 CUs.
//
// SPARSE: the A operand is not dY but the sparsified gradient of the max-gradient approximation (Algorithm 1), built
// from every map's selected position and sum (rounded to bf16, nearest even) while it is written to LDS.
#include <type_traits>
#include "exact_common.hpp"

namespace wgrad {

typedef __bf16 pl_bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t pl_u32x4 __attribute__((ext_vector_type(4)));

struct PlanesParams {
    const void *X[kMaxBatch], *dY[kMaxBatch];
    float *out[kMaxBatch];              // dW of every problem
    const int32_t *hw[kMaxBatch];       // SPARSE: selected position of every map, (row << 16 | col), [N][K]
    const float *sum[kMaxBatch];        // SPARSE: sum of every map, [N][K]
    float scale;                        // applied to what is written
    int per_prob;                       // workgroups per problem
    int N, K, C;
    int bk, bc;                         // tiles of one XCD's block per problem (rows x columns); 0: tiles in plain order
};

constexpr int kPlanesKT = 32;                                   // output channels per workgroup
__host__ __device__ constexpr int planes_ct(int hw) { return hw == 2 ? 64 : 32; }   // input channels per workgroup
__host__ __device__ constexpr size_t planes_lds_bytes(int hw) { return (size_t)2 * hw * hw * (kPlanesKT + planes_ct(hw)) * 32 * 2; }   // two buffers

template <int HW, bool SPARSE>
__device__ __forceinline__ void planes_body(const PlanesParams &p, char *smem, int bid)
{
    constexpr int P = HW * HW;                    // positions of a plane
    constexpr int KT = kPlanesKT, CT = planes_ct(HW);
    constexpr int NTC = CT / 32;                  // 16-column tiles of a wavefront
    constexpr int PV = P < 8 ? P : 8;             // positions per staging task (one 8- or 16-byte load per image)
    constexpr int PCH = P / PV;                   // staging tasks per plane
    constexpr int LW = PV / 2;                    // 32-bit words per load
    typedef uint32_t word;
    // eight wavefronts: four multiply (2 x 2 tiles of the workgroup's result), four stage (loads, transposition,
    // LDS writes); a SIMD holds one of each, so the staging runs under the matrix instructions of the other
    // (a lone wavefront per SIMD overlapped nothing: its stage time was the sum of the parts)
    const int tid = threadIdx.x & (kBlock - 1), lane = tid & 63, wave = tid >> 6;      // tid: number among the staging (or the multiplying) threads
    const bool producer = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 8) != 0;
    const int i16 = lane & 15, kk = lane >> 4;
    const int wk = wave & 1, wc = wave >> 1;

    // Workgroups go to the XCDs round robin.  Every operand row is fetched once per tile column (row) of the result
    // that needs it, out of the XCD's own L2: an XCD therefore takes a block of bk x bc tiles of every problem -- as
    // square as the tile counts allow -- instead of every eighth tile, and fetches bk / (K / 32) of dY and
    // bc / (C / CT) of X instead of all of one of them.
    const int ctiles = p.C / CT;
    int prob, kt, ct;
    if (p.bk) {
        const int xcd = bid & 7, i = bid >> 3, per_xcd = p.bk * p.bc, bcols = ctiles / p.bc;
        prob = i / per_xcd;
        const int tl = i - prob * per_xcd;
        kt = (xcd / bcols) * p.bk + tl / p.bc;
        ct = (xcd % bcols) * p.bc + tl % p.bc;
    } else {
        prob = bid / p.per_prob;
        const int tile = bid - prob * p.per_prob;
        kt = tile / ctiles; ct = tile % ctiles;
    }
    const int k0 = kt * KT, c0 = ct * CT;
    const char *const Xp = (const char *)p.X[prob];
    const char *const dYp = (const char *)p.dY[prob];

    // a buffer: A [P][KT][32] bf16, then B [P][CT][32] bf16; two buffers

    // ---- staging tasks of this thread: (row, group of 8 images, chunk of PV positions) ----
    // A: KT rows x 4 groups x PCH chunks, B: CT rows x 4 groups x PCH chunks; every thread has one of each (on 2x2
    // planes there are only 128 A tasks: the upper half of the workgroup repeats the lower half's, writing the same
    // bytes to the same places, which keeps the loop free of divergent branches)
    constexpr int A_TASKS = KT * 4 * PCH, B_TASKS = CT * 4 * PCH;
    static_assert(kBlock % A_TASKS == 0 && B_TASKS == kBlock, "one staging task of each operand per thread");
    const int ta = tid % A_TASKS;
    const int a_r = ta % KT, a_g = (ta / KT) & 3, a_pc = ta / (KT * 4);
    const int b_r = tid % CT, b_g = (tid / CT) & 3, b_pc = tid / (CT * 4);
    // byte offsets of the first image's piece from the tensor's start; image to image: K (C) planes
    const uint32_t a_src = (uint32_t)((((8 * a_g) * p.K + k0 + a_r) * P + PV * a_pc) * 2);
    const uint32_t b_src = (uint32_t)((((8 * b_g) * p.C + c0 + b_r) * P + PV * b_pc) * 2);
    const uint32_t a_img = (uint32_t)p.K * P * 2, b_img = (uint32_t)p.C * P * 2;
    const uint32_t a_sel = (uint32_t)(((8 * a_g) * p.K + k0 + a_r) * 4);       // SPARSE: offset into hw / sum
    // LDS byte offset (inside a buffer) of the piece of position 0 of the task's chunk; position to position: rows * 64 bytes
    const uint32_t a_dst = (uint32_t)(((PV * a_pc) * KT + a_r) * 64 + 16 * (a_g ^ ((a_r >> 1) & 3)));
    const uint32_t b_dst = (uint32_t)P * KT * 64 + (uint32_t)(((PV * b_pc) * CT + b_r) * 64 + 16 * (b_g ^ ((b_r >> 1) & 3)));

    // two register sets: while the pieces of one stage are transposed into LDS, the next stage's are in flight
    constexpr int AW = SPARSE ? 2 : LW;
    word la[2][8][AW], lb[2][8][LW];              // SPARSE: la = (position word, sum bits) of 8 maps
    auto load_piece = [](word (&dst)[LW], const char *src) {
        if constexpr (LW == 4) {
            const pl_u32x4 v = *(const pl_u32x4 *)src;
            dst[0] = v[0]; dst[1] = v[1]; dst[2] = v[2]; dst[3] = v[3];
        } else {
            const uint2 v = *(const uint2 *)src;
            dst[0] = v.x; dst[1] = v.y;
        }
    };
    auto load_stage = [&](auto set_c, int n0) {
        constexpr int SET = decltype(set_c)::value;
        const uint32_t a_off = (uint32_t)n0 * a_img, b_off = (uint32_t)n0 * b_img;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if constexpr (SPARSE) {
                const uint32_t o = a_sel + (uint32_t)(n0 + j) * (uint32_t)p.K * 4u;
                la[SET][j][0] = (word)*(const int32_t *)((const char *)p.hw[prob] + o);
                la[SET][j][1] = __float_as_uint(*(const float *)((const char *)p.sum[prob] + o));
            } else {
                load_piece(la[SET][j], dYp + a_off + a_src + (uint32_t)j * a_img);
            }
            load_piece(lb[SET][j], Xp + b_off + b_src + (uint32_t)j * b_img);
        }
    };
    // One unit of the transposition: position t of the task's chunk is the same half-word of the 8 images' word
    // t / 2, two images per output word, 16 bytes in all.  SPARSE A: the map's sum, rounded to bf16 (nearest
    // even), where the map's selected position is this one, zero elsewhere.
    auto write_unit = [&](auto set_c, int u, char *buf) {
        constexpr int SET = decltype(set_c)::value;
        pl_u32x4 o;
        if (u < PV) {
            const int t = u;
            if constexpr (SPARSE) {
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    word w = 0;
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        const word hwv = la[SET][2 * d + e][0], sb = la[SET][2 * d + e][1];
                        const int sel = (int)((hwv >> 16) * HW + (hwv & 0xffffu)) - PV * a_pc;
                        const word bf = (sb + 0x7fffu + ((sb >> 16) & 1u)) >> 16;
                        w |= sel == t ? bf << (16 * e) : 0u;
                    }
                    o[d] = w;
                }
            } else {
#pragma unroll
                for (int d = 0; d < 4; ++d)
                    o[d] = __builtin_amdgcn_perm(la[SET][2 * d + 1][t >> 1], la[SET][2 * d][t >> 1], (t & 1) ? 0x07060302u : 0x05040100u);
            }
            *(pl_u32x4 *)(buf + a_dst + (size_t)t * KT * 64) = o;
        } else {
            const int t = u - PV;
#pragma unroll
            for (int d = 0; d < 4; ++d)
                o[d] = __builtin_amdgcn_perm(lb[SET][2 * d + 1][t >> 1], lb[SET][2 * d][t >> 1], (t & 1) ? 0x07060302u : 0x05040100u);
            *(pl_u32x4 *)(buf + b_dst + (size_t)t * CT * 64) = o;
        }
    };

    // ---- operands of this wavefront (byte offsets inside a buffer) ----
    const uint32_t swz = 16u * (uint32_t)(kk ^ ((i16 >> 1) & 3));
    const uint32_t a_rd = (uint32_t)((wk * 16 + i16) * 64) + swz;                                  // + position * KT * 64
    const uint32_t b_rd = (uint32_t)P * KT * 64 + (uint32_t)((wc * (CT / 2) + i16) * 64) + swz;    // + position * CT * 64 + column tile * 16 * 64
    constexpr size_t BUF = planes_lds_bytes(HW) / 2;
    constexpr int UNITS = 2 * PV;                  // transposition units per thread and stage
    static_assert(UNITS % P == 0, "the units of a stage are spread evenly over the positions");
    const int stages = p.N / 32;
    typedef std::integral_constant<int, 0> set0;
    typedef std::integral_constant<int, 1> set1;
    // Stage s is multiplied out of buffer s % 2 while the pieces of stage s + 1 (register set (s + 1) % 2, requested a
    // stage ago) are transposed into the other buffer and the pieces of stage s + 2 are requested into the set that
    // stage s came from; one barrier per stage.  Past the end the last stage is requested and transposed again
    // (never read): the loops are free of branches.  Both kinds of wavefront pass 1 + stages barriers.
    if (producer) {
        auto stage_next = [&](auto par_c, int s) {
            constexpr int PAR = decltype(par_c)::value;
            typedef std::integral_constant<int, PAR> this_set;
            typedef std::integral_constant<int, PAR ^ 1> next_set;
            char *nxt = smem + (PAR ^ 1) * BUF;
            const int s2 = s + 2 < stages ? s + 2 : stages - 1;
            load_stage(this_set{}, 32 * s2);
#pragma unroll
            for (int u = 0; u < UNITS; ++u) write_unit(next_set{}, u, nxt);
            __syncthreads();      // the other buffer is complete; everyone has left this one
        };
        load_stage(set0{}, 0);
#pragma unroll
        for (int u = 0; u < UNITS; ++u) write_unit(set0{}, u, smem);
        load_stage(set1{}, stages > 1 ? 32 : 0);
        __syncthreads();
        int s = 0;
        for (; s + 1 < stages; s += 2) {
            stage_next(set0{}, s);
            stage_next(set1{}, s + 1);
        }
        if (s < stages) stage_next(set0{}, s);
        return;
    }

    float4_t acc[NTC][9];
#pragma unroll
    for (int nt = 0; nt < NTC; ++nt)
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[nt][t] = float4_t{0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](const char *cur) {
        // every position's B operand, then the A operands one by one (each requested a position ahead), each
        // against the taps that stay inside X
        pl_bf16x8 bop[NTC][P];
#pragma unroll
        for (int nt = 0; nt < NTC; ++nt)
#pragma unroll
            for (int q = 0; q < P; ++q) bop[nt][q] = *(const pl_bf16x8 *)(cur + b_rd + (size_t)(q * CT + nt * 16) * 64);
        pl_bf16x8 aop = *(const pl_bf16x8 *)(cur + a_rd);
#pragma unroll
        for (int pp = 0; pp < P; ++pp) {
            pl_bf16x8 aop_next = aop;
            if (pp + 1 < P) aop_next = *(const pl_bf16x8 *)(cur + a_rd + (size_t)(pp + 1) * KT * 64);
            const int h = pp / HW, w = pp % HW;
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int ih = h + t / 3 - 1, iw = w + t % 3 - 1;
                if (ih < 0 || ih >= HW || iw < 0 || iw >= HW) continue;          // the tap lies in the padding
#pragma unroll
                for (int nt = 0; nt < NTC; ++nt)
                    acc[nt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aop, bop[nt][ih * HW + iw], acc[nt][t], 0, 0, 0);
            }
            aop = aop_next;
        }
        __syncthreads();
    };
    __syncthreads();
    for (int s = 0; s < stages; ++s) multiply(smem + (s & 1) * BUF);

    // ---- the nine taps of every (k, c) of the tile: a lane holds rows 4 * kk + v, column i16 of each 16 x 16 tile ----
    float *const out = p.out[prob];
#pragma unroll
    for (int nt = 0; nt < NTC; ++nt)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int k = k0 + wk * 16 + 4 * kk + v, c = c0 + wc * (CT / 2) + nt * 16 + i16;
            float *o = out + ((size_t)k * p.C + c) * 9;
#pragma unroll
            for (int t = 0; t < 9; ++t) o[t] = acc[nt][t][v] * p.scale;
        }
}

template <int HW, bool SPARSE>
__global__ __launch_bounds__(2 * kBlock, 2) void wgrad_exact_bf16_planes(const PlanesParams p)
{
    extern __shared__ char planes_smem[];
    planes_body<HW, SPARSE>(p, planes_smem, (int)blockIdx.x);
}

// Whether the shape is this kernel's (alignment of the tensors is checked at launch).
bool planes_bf16_takes(const Geometry &g)
{
    if (!g.bf16 || g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1) return false;
    if (!((g.H == 2 && g.W == 2) || (g.H == 4 && g.W == 4))) return false;
    if (!tune_int("WGRAD_BF16_PLANES", 1)) return false;
    return g.N % 32 == 0 && g.K % kPlanesKT == 0 && g.C % planes_ct(g.H) == 0
           && (long)g.N * g.K * g.H * g.W * 2 < (1l << 31) && (long)g.N * g.C * g.H * g.W * 2 < (1l << 31);
}

template <int HW, bool SPARSE>
static int planes_launch(const PlanesParams &p, int grid, hipStream_t st)
{
    const size_t lds = planes_lds_bytes(HW);
    if (lds > 64 * 1024 && hipFuncSetAttribute((const void *)wgrad_exact_bf16_planes<HW, SPARSE>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return WGRAD_LAUNCH_FAILED;
    WGRAD_LAUNCH((wgrad_exact_bf16_planes<HW, SPARSE>), dim3((unsigned)grid), dim3(2 * kBlock), lds, st, p);
    return launch_status();
}

// One launch for the whole batch of problems; writes dW itself (no split, no partial sums).  With `sparse` the A
// operand is the sparsified gradient given by every map's selected position and sum.
int launch_exact_bf16_planes(const Geometry &g, const Batch &b, hipStream_t st, const SparseA *sparse)
{
    PlanesParams p{};
    for (int i = 0; i < kMaxBatch; ++i) {
        const int j = i < b.n ? i : 0;
        p.X[i] = b.X[j]; p.dY[i] = b.dY[j]; p.out[i] = b.dW[j];
        p.hw[i] = sparse ? sparse->hw[j] : nullptr;
        p.sum[i] = sparse ? sparse->sum[j] : nullptr;
    }
    p.scale = sparse ? sparse->scale : 1.0f;
    p.N = g.N; p.K = g.K; p.C = g.C;
    const int ktn = g.K / kPlanesKT, ctn = g.C / planes_ct(g.H);
    p.per_prob = ktn * ctn;
    // the block of tiles that one XCD takes of every problem: bk x bc = a eighth of the tiles, eight blocks tiling the result
    p.bk = p.bc = 0;
    if (p.per_prob % 8 == 0 && tune_int("WGRAD_BF16_PLANES_XCD", 1)) {
        const int per_xcd = p.per_prob / 8;
        double best = 1e30;
        for (int bc = 1; bc <= ctn; ++bc) {
            if (ctn % bc || per_xcd % bc) continue;
            const int bk = per_xcd / bc;
            if (bk > ktn || ktn % bk || (ktn / bk) * (ctn / bc) != 8) continue;
            const double cost = (double)bk / ktn + (double)bc / ctn;
            if (cost < best) { best = cost; p.bk = bk; p.bc = bc; }
        }
    }
    const int grid = p.per_prob * b.n;
    if (g.H == 2) return sparse ? planes_launch<2, true>(p, grid, st) : planes_launch<2, false>(p, grid, st);
    return sparse ? planes_launch<4, true>(p, grid, st) : planes_launch<4, false>(p, grid, st);
}

}  // namespace wgrad
