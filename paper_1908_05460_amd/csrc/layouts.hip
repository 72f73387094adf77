// Layout conversions at the library boundary (arXiv 1908.05460, Section 2.4: the paper's kernel reads
// the input channel-last and produces the filter gradient as [C_o,K,K,C_i]; its framework keeps
// NCHW activations and [K,K,C_i,C_o] filters, so it pays an input transpose and a filter-gradient
// transpose around the kernel).  Here both directions of the input transpose, every permutation of
// the filter gradient between OIHW / OHWI / HWIO, and the exact gradient from a channel-last input.
#include "common.hpp"

namespace wgrad {

namespace {

constexpr int kTile = 64;

// dst[b][c][r] = src[b][r][c] for `batch` matrices of rows x cols elements (T = 2- or 4-byte element).
// A workgroup moves one 64 x 64 tile through LDS: rows are read and written along the fastest axis
// of their side; the tile pitch of 65 keeps the column reads free of bank conflicts.
template <typename T>
__global__ __launch_bounds__(kBlock) void transpose_batched(const T *__restrict__ src, T *__restrict__ dst,
                                                            int rows, int cols, int tiles_c, int tiles_r)
{
    __shared__ T tile[kTile][kTile + 1];
    const int t = blockIdx.x % (tiles_c * tiles_r);
    const long b = blockIdx.x / (tiles_c * tiles_r);
    const int r0 = (t / tiles_c) * kTile, c0 = (t % tiles_c) * kTile;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const T *s = src + b * (long)rows * cols;
    T *d = dst + b * (long)rows * cols;
#pragma unroll 4
    for (int i = wave; i < kTile; i += kBlock / 64) {
        const int r = r0 + i, c = c0 + lane;
        if (r < rows && c < cols) tile[i][lane] = s[(long)r * cols + c];
    }
    __syncthreads();
#pragma unroll 4
    for (int i = wave; i < kTile; i += kBlock / 64) {
        const int c = c0 + i, r = r0 + lane;
        if (r < rows && c < cols) d[(long)c * rows + r] = tile[lane][i];
    }
}

// One thread per element of the destination; the filter gradient is small (at most a few MB).
__global__ __launch_bounds__(kBlock) void permute_dw(const float *__restrict__ src, float *__restrict__ dst,
                                                     int K, int C, int R, int S, int from, int to)
{
    const long o = (long)blockIdx.x * kBlock + threadIdx.x;
    const long total = (long)K * C * R * S;
    if (o >= total) return;
    int k, c, r, s;
    long q = o;
    if (to == WGRAD_DW_OHWI)      { c = q % C; q /= C; s = q % S; q /= S; r = q % R; k = (int)(q / R); }
    else if (to == WGRAD_DW_HWIO) { k = q % K; q /= K; c = q % C; q /= C; s = q % S; r = (int)(q / S); }
    else                          { s = q % S; q /= S; r = q % R; q /= R; c = q % C; k = (int)(q / C); }
    long at;
    if (from == WGRAD_DW_OHWI)      at = (((long)k * R + r) * S + s) * C + c;
    else if (from == WGRAD_DW_HWIO) at = (((long)r * S + s) * C + c) * K + k;
    else                            at = (((long)k * C + c) * R + r) * S + s;
    dst[o] = src[at];
}

int launch_transpose(const void *src, void *dst, long batch, int rows, int cols, bool two_byte, hipStream_t st)
{
    const int tc = (cols + kTile - 1) / kTile, tr = (rows + kTile - 1) / kTile;
    const long blocks = batch * tc * tr;
    if (blocks >= (1l << 31)) return WGRAD_UNSUPPORTED;
    if (two_byte)
        WGRAD_LAUNCH((transpose_batched<uint16_t>), dim3((unsigned)blocks), dim3(kBlock), 0, st,
                     (const uint16_t *)src, (uint16_t *)dst, rows, cols, tc, tr);
    else
        WGRAD_LAUNCH((transpose_batched<uint32_t>), dim3((unsigned)blocks), dim3(kBlock), 0, st,
                     (const uint32_t *)src, (uint32_t *)dst, rows, cols, tc, tr);
    return launch_status();
}

}  // namespace

bool dw_layout_ok(int layout)
{
    return layout == WGRAD_DW_OIHW || layout == WGRAD_DW_OHWI || layout == WGRAD_DW_HWIO;
}

int launch_transpose_x(const Geometry &g, bool to_nhwc, const void *src, void *dst, hipStream_t st)
{
    // per image: [C][H*W] -> [H*W][C], or back
    const int HW = g.H * g.W;
    return to_nhwc ? launch_transpose(src, dst, g.N, g.C, HW, g.bf16, st)
                   : launch_transpose(src, dst, g.N, HW, g.C, g.bf16, st);
}

int launch_permute_dw(const Geometry &g, int from, int to, const float *src, float *dst, hipStream_t st)
{
    const long total = g.dw_elems();
    WGRAD_LAUNCH(permute_dw, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, st,
                 src, dst, g.K, g.C, g.R, g.S, from, to);
    return launch_status();
}

// Exact gradient from a channel-last input: the input is brought to NCHW in the workspace, the
// NCHW kernels run on it, and the result is permuted into the requested layout.
// Workspace: [X as NCHW][dW as OIHW, unless that is the requested layout][the exact path's own].
size_t exact_nhwc_ws_bytes(const Geometry &g, const ExactPlan &pl)
{
    return align_up((size_t)g.N * g.C * g.H * g.W * (g.bf16 ? 2 : 4)) + align_up((size_t)g.dw_elems() * 4) +
           align_up(pl.ws_bytes);
}

int launch_exact_nhwc(const Geometry &g, const ExactPlan &pl, const void *X, const void *dY, float *dW,
                      int dw_layout, void *ws, hipStream_t st)
{
    char *w = (char *)ws;
    void *Xt = w;              w += align_up((size_t)g.N * g.C * g.H * g.W * (g.bf16 ? 2 : 4));
    float *tmp = (float *)w;   w += align_up((size_t)g.dw_elems() * 4);
    int rc = launch_transpose_x(g, /*to_nhwc=*/false, X, Xt, st);
    if (rc != WGRAD_OK) return rc;
    Batch b{};
    b.n = 1; b.X[0] = Xt; b.dY[0] = dY; b.dW[0] = dw_layout == WGRAD_DW_OIHW ? dW : tmp;
    rc = launch_exact(g, pl, b, w, st);
    if (rc != WGRAD_OK || dw_layout == WGRAD_DW_OIHW) return rc;
    return launch_permute_dw(g, WGRAD_DW_OIHW, dw_layout, tmp, dW, st);
}

}  // namespace wgrad
