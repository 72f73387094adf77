// Instantiations of the streaming exact-gradient kernel for K tiles of 64 output channels.

#include "exact_stream_kernel.hpp"

namespace wgrad {

void stream_launch_w4(const StreamParams &p, int nt, int xv, int gpw, int rowp, int grid, size_t lds, hipStream_t st)
{
    if (p.s.g.bf16) stream_pick<4, true>(p, nt, xv, gpw, rowp, grid, lds, st);
    else stream_pick<4, false>(p, nt, xv, gpw, rowp, grid, lds, st);
}








}  // namespace wgrad
