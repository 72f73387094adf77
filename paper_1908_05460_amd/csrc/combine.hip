// Reduction of partial results: dW[o] = scale * sum_j partial[j][o], for a table of tensors in
// one launch.  The split reductions of the exact kernel and the batch chunks of the approximated
// one both end here.
#include <algorithm>

#include "common.hpp"

namespace wgrad {

struct CombineTable {
    int n;
    int begin[kTableMax + 1];        // first workgroup of each tensor; begin[n] = grid size
    CombineItem item[kTableMax];
    unsigned char pl_log[kTableMax]; // log2 of the lanes that share one output; kVec4: one lane, four outputs
};
constexpr int kVec4 = 8;

// PL = 2^pl_log lanes share one output: lane pl adds partials pl, pl+PL, ... in ascending order,
// then the PL sub-sums are added in ascending pl through LDS -- a fixed order, so the result is
// deterministic.  PL > 1 spreads a long list of partials of a small tensor over more lanes.
__global__ __launch_bounds__(kBlock) void combine_table(const CombineTable t)
{
    __shared__ float red[kBlock];
    int it = 0;
    for (int i = 1; i < t.n; ++i) it += (int)blockIdx.x >= t.begin[i];
    const CombineItem c = t.item[it];
    if (t.pl_log[it] == kVec4) {
        // large tensors: four consecutive outputs per lane, 16-byte accesses (elems % 4 == 0, pointers 16-byte aligned)
        const long o = ((long)((int)blockIdx.x - t.begin[it]) * kBlock + threadIdx.x) * 4;
        if (o >= c.elems) return;
        const float *__restrict__ part = c.part;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        int i = 0;
        for (; i + 3 < c.nparts; i += 4) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *(const float4 *)(part + (long)(i + u) * c.elems + o);
#pragma unroll
            for (int u = 0; u < 4; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
        }
        for (; i < c.nparts; ++i) {
            const float4 v = *(const float4 *)(part + (long)i * c.elems + o);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *(float4 *)(c.dW + o) = make_float4(acc.x * c.scale, acc.y * c.scale, acc.z * c.scale, acc.w * c.scale);
        return;
    }
    const int lg = t.pl_log[it];
    const int PL = 1 << lg, OB = kBlock >> lg;          // outputs per workgroup
    const int ol = threadIdx.x & (OB - 1), pl = threadIdx.x >> (8 - lg);
    const long o = (long)((int)blockIdx.x - t.begin[it]) * OB + ol;
    const float *__restrict__ part = c.part;
    const long elems = c.elems;
    float acc = 0.f;
    if (o < elems) {
        int i = pl;
        for (; i + 7 * PL < c.nparts; i += 8 * PL) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(long)(i + u * PL) * elems + o];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (; i < c.nparts; i += PL) acc += part[(long)i * elems + o];
    }
    if (lg == 0) {
        if (o < elems) c.dW[o] = acc * c.scale;
        return;
    }
    red[pl * OB + ol] = acc;
    __syncthreads();
    if (pl == 0 && o < elems) {
        float s = 0.f;
        for (int q = 0; q < PL; ++q) s += red[q * OB + ol];
        c.dW[o] = s * c.scale;
    }
}

int combine_flush(CombineQueue &q, hipStream_t st)
{
    for (size_t first = 0; first < q.item.size(); first += kTableMax) {
        const int n = (int)std::min<size_t>(kTableMax, q.item.size() - first);
        CombineTable t{};
        t.n = n;
        int blocks = 0;
        for (int i = 0; i < n; ++i) {
            const CombineItem &c = q.item[first + i];
            // spread the partial index over lanes when there are few outputs and many partials
            int lg = (c.elems <= 16 * 1024 && c.nparts >= 64) ? 4 : ((c.elems <= 256 * 1024 && c.nparts >= 16) ? 2 : 0);
            int ob = kBlock >> lg;
            if (lg == 0 && c.elems >= 64 * 1024 && c.elems % 4 == 0 && ((uintptr_t)c.part % 16) == 0 && ((uintptr_t)c.dW % 16) == 0) {
                lg = kVec4;
                ob = kBlock * 4;
            }
            t.item[i] = c;
            t.pl_log[i] = (unsigned char)lg;
            t.begin[i] = blocks;
            blocks += (c.elems + ob - 1) / ob;
        }
        t.begin[n] = blocks;
        WGRAD_LAUNCH(combine_table, dim3((unsigned)blocks), dim3(kBlock), 0, st, t);
        if (launch_status() != WGRAD_OK) { q.item.clear(); return WGRAD_LAUNCH_FAILED; }
    }
    q.item.clear();
    return WGRAD_OK;
}

int launch_combine(const float *partials, long prob_stride, int nparts, long elems, float scale,
                   float *const *dW, int nprob, hipStream_t st, CombineQueue *defer)
{
    CombineQueue local;
    CombineQueue &q = defer ? *defer : local;
    if (elems >= (1l << 31)) return WGRAD_UNSUPPORTED;        // a table entry counts its elements in an int
    for (int i = 0; i < nprob; ++i)
        q.item.push_back(CombineItem{partials + i * prob_stride, dW[i], nparts, (int)elems, scale});
    return defer ? WGRAD_OK : combine_flush(local, st);
}

}  // namespace wgrad
