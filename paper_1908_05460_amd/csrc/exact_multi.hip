// One launch for several layer shapes of the exact filter gradient (fp32 inputs).  A run over a
// whole network launches one streaming kernel per group of identical layers; on small networks each
// of those launches pays its ramp (every workgroup fetching its first window at once), its tail and
// the gap to the next launch with most of the chip idle.  Here the workgroups of up to kMultiMax
// groups are one grid: a workgroup looks up its group, then runs that group's instantiation of the
// streaming body.  Workgroups of different groups share the CUs, so one group's ramp and tail hide
// under the others' matrix work, and each group can be cut into fewer, longer workgroups.
#define WGRAD_TRACE_HERE
#include "exact_plane2_kernel.hpp"

namespace wgrad {

struct MultiParams {
    int n;
    int begin[kMultiMax + 1];       // first workgroup of each group (multiples of 8: the XCD numbering of a
                                    // group then starts on XCD 0); begin[n] = grid size
    int count[kMultiMax];           // workgroups of the group that do work (the rest of its share exit)
    int variant[kMultiMax];
    int first[kMultiMax];           // the group's first problem in the tensor tables
    StreamShape s[kMultiMax];
    const void *X[kMultiTensors], *dY[kMultiTensors];
    float *out[kMultiTensors];
};
static_assert(sizeof(MultiParams) <= 4096, "kernel arguments");

// The instantiations a multi-shape launch can mix: 3x3 layers of CIFAR-sized networks (maps of 32, 16, 8, 4,
// 2 and the first layer's three input channels).  (NT, WK, XV, GPW, ROWP)
#define WGRAD_MULTI_VARIANTS(X) \
    X(0, 2, 1, 4, 8, 0, 0, false)  X(1, 9, 1, 4, 4, 36, 0, false) X(2, 9, 2, 4, 2, 36, 0, false) X(3, 9, 2, 4, 8, 20, 0, false)  \
    X(4, 9, 4, 4, 4, 20, 0, false) X(5, 9, 4, 4, 8, 12, 0, false) X(6, 2, 4, 4, 8, 0, 0, false)  X(7, 9, 4, 4, 8, 36, 0, false)  \
    X(8, 9, 4, 4, 8, 20, 0, false) X(9, 9, 4, 4, 4, 12, 0, false) X(10, 9, 4, 2, 4, 4, 0, false) X(12, 9, 4, 4, 4, 12, 1, false) \
    X(13, 9, 4, 4, 8, 12, 2, false) X(14, 9, 4, 4, 8, 20, 4, false) X(15, 9, 4, 4, 8, 36, 8, false) \
    X(16, 9, 2, 4, 8, 20, 4, false) X(17, 9, 4, 4, 8, 6, 1, true)

constexpr int kMultiPlane2 = 11;    // the 2x2-plane matrix-product form rides along as one more variant

int multi_variant(int nt, int wk, int xv, int gpw, int rowp, int wc, int img4)
{
#define X(ID, NT, WK, XV, GPW, ROWP, WC, IMG4) if (nt == NT && wk == WK && xv == XV && gpw == GPW && rowp == ROWP && wc == WC && (img4 != 0) == IMG4) return ID;
    WGRAD_MULTI_VARIANTS(X)
#undef X
    return -1;
}

// The parameters are read through the kernel-argument segment pointer: indexing the by-value argument
// with a run-time group number would make the compiler copy all of it into scratch memory first.
__global__ __launch_bounds__(kBlock, 3) void wgrad_exact_multi(const MultiParams)
{
    extern __shared__ float smem[];
    const MultiParams *mp = (const MultiParams *)__builtin_amdgcn_kernarg_segment_ptr();
    const int n = mp->n;
    int gi = 0;
    for (int i = 1; i < n; ++i) gi += (int)blockIdx.x >= mp->begin[i];
    const int bid = (int)blockIdx.x - mp->begin[gi], nblk = mp->count[gi];
    if (bid >= nblk) return;
    const StreamShape &p = mp->s[gi];       // still kernel-argument memory at a uniform address: scalar loads
    const int first = mp->first[gi];
    const void *const *Xt = mp->X + first, *const *dYt = mp->dY + first;
    float *const *outt = mp->out + first;
    switch (mp->variant[gi]) {
#define X(ID, NT, WK, XV, GPW, ROWP, WC, IMG4) case ID: stream_body<NT, WK, false, XV, GPW, ROWP, WC, IMG4>(p, Xt, dYt, outt, smem, bid, nblk); break;
        WGRAD_MULTI_VARIANTS(X)
#undef X
        case kMultiPlane2: plane2_body(p, Xt, dYt, outt, bid); break;
        default: break;
    }
}

int multi_flush(MultiQueue &q, hipStream_t st)
{
    if (q.n == 0) return WGRAD_OK;
    int rc = WGRAD_OK;
    if (q.n == 1) {
        const StreamLaunch &L = q.item[0];
        rc = launch_stream_now(L, st);
        q.n = 0; q.tensors = 0;
        return rc;
    }
    MultiParams mp{};
    mp.n = q.n;
    size_t lds = 0;
    int blocks = 0, tensors = 0;
    for (int i = 0; i < q.n; ++i) {
        const StreamLaunch &L = q.item[i];
        mp.begin[i] = blocks;
        mp.count[i] = L.grid;
        mp.variant[i] = L.plane2 ? kMultiPlane2 : multi_variant(L.nt, L.wk, L.xv, L.gpw, L.rowp_inst, L.wc, L.img4);
        mp.s[i] = L.p.s;
        mp.first[i] = tensors;
        for (int j = 0; j < L.nprob; ++j, ++tensors) { mp.X[tensors] = L.p.X[j]; mp.dY[tensors] = L.p.dY[j]; mp.out[tensors] = L.p.out[j]; }
        blocks += (L.grid + 7) / 8 * 8;
        if (L.lds > lds) lds = L.lds;
    }
    mp.begin[q.n] = blocks;
    q.n = 0; q.tensors = 0;
    WGRAD_LAUNCH(wgrad_exact_multi, dim3((unsigned)blocks), dim3(kBlock), lds, st, mp);
    return launch_status();
}


}  // namespace wgrad

WGRAD_TRACE_READER(wgrad_debug_read_trace_multi)
