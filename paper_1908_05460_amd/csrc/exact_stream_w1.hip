// Instantiations of the streaming exact-gradient kernel for K tiles of 16 output channels.
#define WGRAD_TRACE_HERE
#include "exact_stream_kernel.hpp"

namespace wgrad {

void stream_launch_w1(const StreamParams &p, int nt, int xv, int gpw, int rowp, int grid, size_t lds, hipStream_t st)
{
    if (p.g.bf16) stream_pick<1, true>(p, nt, xv, gpw, rowp, grid, lds, st);
    else stream_pick<1, false>(p, nt, xv, gpw, rowp, grid, lds, st);
}

#if defined(WGRAD_TUNING) && !defined(WGRAD_NO_TRACE)
extern "C" int wgrad_debug_read_trace(long long *host_out)
{
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_trace), sizeof(long long) * (64 + 2 * 4096));
}
#endif

}  // namespace wgrad
