/*
 * wgrad.h - C ABI of libwgrad: the filter (weight) gradient of a convolution
 * layer on AMD MI355X (gfx950), exact and in the approximated forms of
 * "Accelerated CNN Training Through Gradient Approximation" (arXiv 1908.05460).
 *
 * Tensors (Section 2.4 states the layer in NCHW; the paper's I, dO, df, C_i, C_o
 * and filter size K are X, dY, dW, C, K and R x S here):
 *   X   [N,C,H,W]      input activations saved by the forward pass, contiguous
 *   dY  [N,K,Ho,Wo]    gradient w.r.t. the layer output, contiguous
 *   dW  [K,C,R,S]      gradient w.r.t. the filters, contiguous, always float32
 *   Ho = floor((H + 2*pad_h - R)/stride_h) + 1,  Wo likewise.
 *
 * Conventions for every entry point
 *   - All tensor and workspace pointers are DEVICE pointers owned by the caller
 *     (256-byte aligned workspace; tensors aligned to their element size; 16-byte
 *     alignment enables the vector paths).  Descriptors and per-layer pointer
 *     tables are HOST memory and are read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; they never allocate, free or synchronise.
 *   - dW is OVERWRITTEN, never accumulated into (Algorithm 1 starts from df = 0).
 *   - Return value: WGRAD_OK (0) or a negative wgrad_status.  All validation is
 *     done on the host before anything is launched, so on error nothing was
 *     enqueued by that call.
 *   - Thread-safe for calls that use distinct workspaces; calls sharing a
 *     workspace must be ordered on one stream.
 */
#ifndef WGRAD_H
#define WGRAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t N, C, H, W;          /* X  : [N,C,H,W]                                   */
    int32_t K, R, S;             /* dW : [K,C,R,S]                                   */
    int32_t stride_h, stride_w;  /* >= 1                                             */
    int32_t pad_h, pad_w;        /* >= 0, zero padding                               */
    int32_t dtype;               /* element type of X and dY: WGRAD_F32 or WGRAD_BF16 */
} wgrad_conv_desc;

enum { WGRAD_F32 = 0, WGRAD_BF16 = 1 };

typedef enum { WGRAD_EXACT = 0, WGRAD_APPROX = 1, WGRAD_ZERO = 2, WGRAD_RANDOM = 3 } wgrad_method;

typedef enum {
    WGRAD_OK = 0,
    WGRAD_INVALID_ARG = -1,         /* null pointer, non-positive size, empty output, bad dtype/method */
    WGRAD_UNSUPPORTED = -2,         /* sizes beyond the kernels' 32-bit index ranges; topk out of range */
    WGRAD_WORKSPACE_TOO_SMALL = -3, /* ws_bytes < conv_wgrad_workspace_bytes(), or ws misaligned      */
    WGRAD_LAUNCH_FAILED = -4,       /* the HIP runtime refused a launch                               */
    WGRAD_SCRATCH_LIMIT = -5        /* conv_wgrad_approx_static: the layer needs more than the static buffer */
} wgrad_status;

/* Exact filter gradient (Section 2: the third convolution of a layer's
 * forward-backward pass; Section 2.4: "convolve I with dO"):
 *   dW[k,c,r,s] = sum_{n,h,w} dY[n,k,h,w] * X[n,c,h*stride_h + r - pad_h, w*stride_w + s - pad_w]
 * with X read as zero outside its bounds.  fp32 accumulation for both dtypes.
 * ws: device scratch of at least conv_wgrad_workspace_bytes(desc, WGRAD_EXACT). */
int conv_wgrad_exact(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                     void *ws, size_t ws_bytes, void *stream);

/* Max Gradient Approximation (Section 2.3 and Algorithm 1).  For every map
 * dY[n,k,:,:] keep only the position p* = argmax |dY| (lowest flat index
 * h*Wo + w among equal magnitudes), let it carry the map's signed sum S, and
 * accumulate the input patch that position sees:
 *   dW[k,c,r,s] = scale * sum_n S[n,k] * X[n,c,h* * stride_h + r - pad_h, w* * stride_w + s - pad_w]
 * scale = 1 is Algorithm 1 as printed; the paper's runs use 1/128 (Section 2.3).
 * idx_out, sum_out: optional device arrays of N*K elements (index n*K + k) that
 * receive p* and S; either may be NULL.
 * ws: at least conv_wgrad_workspace_bytes(desc, WGRAD_APPROX). */
int conv_wgrad_approx(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                      float scale, int32_t *idx_out, float *sum_out,
                      void *ws, size_t ws_bytes, void *stream);

/* conv_wgrad_approx for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 * Same arguments, same kernels and same results as conv_wgrad_approx, but the scratch
 * memory is a buffer of WGRAD_STATIC_SCRATCH_BYTES inside the library's device image:
 * each GPU the library runs on holds it from the first call there until the process
 * ends.  The call allocates and frees nothing.  The stream's device must be the current
 * device; the first call on a device looks the buffer's address up (a runtime query, so
 * make that call outside a graph capture).
 * A layer with conv_wgrad_workspace_bytes(desc, WGRAD_APPROX) above the limit is refused
 * with WGRAD_SCRATCH_LIMIT and nothing is launched (24 MiB hold every layer of the CIFAR
 * ResNet-20 and VGG-19 stacks up to batch 512).
 * All calls on one GPU share that GPU's buffer: calls that may overlap in time (different
 * streams, or different host threads) race on it and must be ordered by the caller. */
#define WGRAD_STATIC_SCRATCH_BYTES (24u << 20)
int conv_wgrad_approx_static(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                             float scale, int32_t *idx_out, float *sum_out, void *stream);

/* The two selection quantities of Algorithm 1 alone (its argmax and sum lines):
 * idx[n*K + k] and sum[n*K + k] for every map of dY.  X is not read; only the
 * output geometry of desc matters.  Needs no workspace. */
int conv_wgrad_select(const wgrad_conv_desc *desc, const void *dY, int32_t *idx, float *sum,
                      void *stream);

/* Top-k form of the approximation (Section 2.3 names keeping more than the
 * maximum as the natural refinement; it fixes no weighting, this library's is
 * stated here).  Every map dY[n,k,:,:] keeps its topk positions of largest
 * magnitude, ranked by magnitude descending and by flat index ascending among
 * equal magnitudes; each kept position carries S/topk, S the map's signed sum:
 *   dW[k,c,r,s] = scale * sum_n (S[n,k]/topk) * sum_{j<topk} X[n,c,h_j*stride_h + r - pad_h, w_j*stride_w + s - pad_w]
 * topk = 1 is conv_wgrad_approx.  1 <= topk <= min(64, Ho*Wo), otherwise
 * WGRAD_UNSUPPORTED and nothing is launched.
 * idx_out: optional, N*K*topk elements, idx_out[(n*K + k)*topk + j] = the flat
 * position of rank j; sum_out: optional, N*K elements.
 * ws: at least conv_wgrad_topk_workspace_bytes(desc, topk), 256-byte aligned. */
int conv_wgrad_approx_topk(const wgrad_conv_desc *desc, const void *X, const void *dY, float *dW,
                           int topk, float scale, int32_t *idx_out, float *sum_out,
                           void *ws, size_t ws_bytes, void *stream);

/* Scratch bytes conv_wgrad_approx_topk needs; 0 for an invalid descriptor or topk. */
size_t conv_wgrad_topk_workspace_bytes(const wgrad_conv_desc *desc, int topk);

/* ---- The layouts of the paper's own kernel (Section 2.4, its last paragraphs) ----
 * The paper's kernel reads the input activations channel-last, X[n,h,w,c] (the patch
 * of a selected position is then R rows of S*C contiguous values, and neighbouring
 * threads read neighbouring channels), takes dY as [n,k,h,w] unchanged, and produces
 * the filter gradient as [C_o,K,K,C_i] = dW[k,r,s,c] (OHWI).  Its framework holds
 * activations as NCHW and filters as [K,K,C_i,C_o] = dW[r,s,c,k] (HWIO), so it pays
 * one transpose of X and one of dW around the kernel.  The calls below take X
 * channel-last and write dW in any of the three layouts; the two transposes are
 * also callable on their own so that their cost can be measured. */
typedef enum { WGRAD_DW_OIHW = 0, WGRAD_DW_OHWI = 1, WGRAD_DW_HWIO = 2 } wgrad_dw_layout;

/* conv_wgrad_approx with X given as [N,H,W,C] (element type desc->dtype); dY, idx_out,
 * sum_out as there.  dW (K*C*R*S floats) is written in dw_layout.  Same values as
 * conv_wgrad_approx on the NCHW copy of X, up to the order of the fp32 sums.
 * ws: at least conv_wgrad_nhwc_workspace_bytes(desc, WGRAD_APPROX). */
int conv_wgrad_approx_nhwc(const wgrad_conv_desc *desc, const void *X_nhwc, const void *dY, float *dW,
                           wgrad_dw_layout dw_layout, float scale, int32_t *idx_out, float *sum_out,
                           void *ws, size_t ws_bytes, void *stream);

/* conv_wgrad_exact with X given as [N,H,W,C]: X is transposed to NCHW inside the
 * workspace, the NCHW kernels run, and the result is permuted into dw_layout.
 * ws: at least conv_wgrad_nhwc_workspace_bytes(desc, WGRAD_EXACT). */
int conv_wgrad_exact_nhwc(const wgrad_conv_desc *desc, const void *X_nhwc, const void *dY, float *dW,
                          wgrad_dw_layout dw_layout, void *ws, size_t ws_bytes, void *stream);

/* Scratch bytes of the two calls above; 0 for an invalid descriptor or method. */
size_t conv_wgrad_nhwc_workspace_bytes(const wgrad_conv_desc *desc, wgrad_method method);

/* The paper's input transpose: dst = X as [N,H,W,C] from src = X as [N,C,H,W]
 * (to_nhwc != 0), or the reverse (to_nhwc == 0).  N*C*H*W elements of desc->dtype
 * each; src and dst must not overlap. */
int conv_wgrad_transpose_x(const wgrad_conv_desc *desc, int to_nhwc, const void *src, void *dst, void *stream);

/* The paper's filter-gradient transpose (OHWI -> HWIO) and every other permutation
 * between the three layouts: dst (layout `to`) = src (layout `from`), K*C*R*S floats
 * each; src and dst must not overlap. */
int conv_wgrad_permute_dw(const wgrad_conv_desc *desc, wgrad_dw_layout from, wgrad_dw_layout to,
                          const float *src, float *dst, void *stream);

/* Zero gradient (Section 2.1): dW = 0. */
int conv_wgrad_zero(const wgrad_conv_desc *desc, float *dW, void *stream);

/* Random gradient (Section 2.2): independent N(0, sigma) values (paper: 1/128).
 * dW[i] is a pure function of (seed, offset + i).  With g = offset + i, c = g / 4,
 * j = g mod 4: Philox4x32-10 with counter (lo32, hi32, 0, 0) of c and key
 * (lo32, hi32) of seed gives four words; words (0,1) serve j = 0,1 and words (2,3)
 * serve j = 2,3 as Box-Muller pairs, u = ((word >> 8) + 0.5) / 2^24:
 *   dW[i] = sigma * sqrt(-2 ln u1) * (j even ? cos(2 pi u2) : sin(2 pi u2)).
 * The caller advances offset by K*C*R*S per layer and batch so that every batch
 * draws new numbers, as the method requires. */
int conv_wgrad_random(const wgrad_conv_desc *desc, float *dW, float sigma,
                      uint64_t seed, uint64_t offset, void *stream);

/* Bytes of device scratch the given method needs for this layer (0 for
 * WGRAD_ZERO and WGRAD_RANDOM).  Returns 0 for an invalid descriptor too; use a
 * compute call to learn why a descriptor is rejected. */
size_t conv_wgrad_workspace_bytes(const wgrad_conv_desc *desc, wgrad_method method);

/* One batch of an approximation schedule (Section 2.5): layer i uses
 * method[i] (a wgrad_method).  layers, X, dY, dW and method are host arrays of
 * nlayers entries (at most 4096); X[i], dY[i], dW[i] are device pointers, and
 * the dW tensors must not overlap one another.  All layers are enqueued on
 * `stream` without any host synchronisation, in this order: exact and
 * approximated layers, where those that share one descriptor (up to 8) are
 * folded into one group and up to six groups into a single launch; one
 * reduction of all their partial results; one launch for the zero layers and
 * one for the random layers (32 tensors per launch).  Every layer works in its own slice of `ws`, which must hold
 * conv_wgrad_schedule_workspace_bytes(layers, method, nlayers): the sum over
 * the layers, not their maximum.  The results are those of the individual
 * calls.  A random layer i uses offset + (sum of K*C*R*S of the layers before
 * it).  Validation of every layer happens before the first launch. */
int conv_wgrad_schedule_run(const wgrad_conv_desc *layers, const void *const *X,
                            const void *const *dY, float *const *dW, const uint8_t *method,
                            int32_t nlayers, float scale, float sigma, uint64_t seed,
                            uint64_t offset, void *ws, size_t ws_bytes, void *stream);

size_t conv_wgrad_schedule_workspace_bytes(const wgrad_conv_desc *layers, const uint8_t *method,
                                           int32_t nlayers);

/* conv_wgrad_schedule_run with the top-k form of the approximation (Section 2.3; see
 * conv_wgrad_approx_topk) on the layers whose method is WGRAD_APPROX: every such
 * layer keeps min(topk, Ho*Wo) positions per map.  1 <= topk <= 64, otherwise
 * WGRAD_UNSUPPORTED.  Approximated layers of one shape are folded into a group
 * (and groups into launches) where the fused top-k kernel takes the shape, and
 * run one by one otherwise; everything else is as in conv_wgrad_schedule_run.
 * ws: at least conv_wgrad_schedule_topk_workspace_bytes(layers, method, nlayers, topk). */
int conv_wgrad_schedule_run_topk(const wgrad_conv_desc *layers, const void *const *X,
                                 const void *const *dY, float *const *dW, const uint8_t *method,
                                 int32_t nlayers, int32_t topk, float scale, float sigma,
                                 uint64_t seed, uint64_t offset, void *ws, size_t ws_bytes,
                                 void *stream);

/* Scratch bytes of the call above; 0 for invalid arguments. */
size_t conv_wgrad_schedule_topk_workspace_bytes(const wgrad_conv_desc *layers, const uint8_t *method,
                                                int32_t nlayers, int32_t topk);

/* Static, NUL-terminated description of a status code. */
const char *conv_wgrad_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* WGRAD_H */
