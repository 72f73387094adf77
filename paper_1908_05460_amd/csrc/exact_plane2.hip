// Host side of the 2x2-plane exact-gradient kernel (see exact_plane2_kernel.hpp), and its own launch.
#include "exact_plane2_kernel.hpp"

namespace wgrad {

__global__ __launch_bounds__(kBlock, 2) void wgrad_exact_plane2(const StreamParams p)
{
    plane2_body(p.s, p.X, p.dY, p.out, (int)blockIdx.x);
}

// Whether the shape is this kernel's (alignment of the tensors is checked at launch).
bool plane2_takes(const Geometry &g)
{
    return !g.bf16 && g.H == 2 && g.W == 2 && g.R == 3 && g.S == 3 && g.sh == 1 && g.sw == 1 && g.ph == 1 && g.pw == 1
           && g.K % 16 == 0 && g.C % 16 == 0 && (long)g.N * g.K * 16 < (1l << 32) && (long)g.N * g.C * 16 < (1l << 32);
}

// One launch for the whole batch, or (with a queue) one group of a multi-shape launch.  No split, no partial sums.
int launch_exact_plane2(const Geometry &g, const Batch &b, hipStream_t st, MultiQueue *mq)
{
    StreamLaunch L{};
    StreamShape &p = L.p.s;
    for (int i = 0; i < kMaxBatch; ++i) {
        const int j = i < b.n ? i : 0;
        L.p.X[i] = b.X[j]; L.p.dY[i] = b.dY[j]; L.p.out[i] = b.dW[j];
    }
    L.nprob = b.n;
    p.g = g;
    const int tiles = (g.K / 16) * (g.C / 16);
    p.per_prob = (tiles + kBlock / 64 - 1) / (kBlock / 64);
    L.plane2 = 1;
    L.grid = p.per_prob * b.n;
    if (mq) {
        if (mq->n >= tune_int("WGRAD_MULTI_GROUPS", kMultiMax) || mq->tensors + b.n > kMultiTensors) {
            const int rc = multi_flush(*mq, st);
            if (rc != WGRAD_OK) return rc;
        }
        mq->item[mq->n++] = L;
        mq->tensors += b.n;
        return WGRAD_OK;
    }
    return launch_stream_now(L, st);
}

void launch_plane2_kernel(const StreamLaunch &L, hipStream_t st)
{
    WGRAD_LAUNCH(wgrad_exact_plane2, dim3((unsigned)L.grid), dim3(kBlock), 0, st, L.p);
}

}  // namespace wgrad
