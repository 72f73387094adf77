// DEVELOPMENT BUILDS ONLY (-DWGRAD_TUNING): run-time overrides of the tuning constants and timestamp traces of
// workgroup lifetimes.  The product library is built without WGRAD_TUNING and never includes this file; nothing
// declared here is part of the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdlib.h>

namespace wgrad {

// a tuning constant that an environment variable of the same name may override
inline int tune_int(const char *name, int dflt)
{
    if (const char *v = getenv(name)) return atoi(v);
    return dflt;
}

// A translation unit that wants timestamps defines WGRAD_TRACE_HERE (exact kernels: phases of one workgroup and
// start/end of every workgroup) or WGRAD_TRACE_FUSED_HERE (fused approximation kernel: four marks per workgroup)
// before its first include, and WGRAD_TRACE_READER(name) once at file scope to export a host reader.
#if defined(WGRAD_TRACE_HERE) && !defined(WGRAD_NO_TRACE)
static __device__ long long g_trace[64 + 2 * 4096];
#define TRACE_BLOCK 37
#define TRACE_BLK(which) do { if (threadIdx.x == 0 && blockIdx.x < 4096) g_trace[64 + 2 * blockIdx.x + which] = wall_clock64(); } while (0)
#define TRACE(i) do { if (blockIdx.x == TRACE_BLOCK && threadIdx.x == 0) { g_trace[i] = wall_clock64(); g_trace[32 + i] = clock64(); } } while (0)
#define WGRAD_TRACE_READER(name) \
    extern "C" int name(long long *host_out) { return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(::wgrad::g_trace), sizeof(long long) * (64 + 2 * 4096)); }
#else
#define TRACE(i) do { } while (0)
#define TRACE_BLK(which) do { } while (0)
#define WGRAD_TRACE_READER(name)
#endif

#if defined(WGRAD_TRACE_FUSED_HERE) && !defined(WGRAD_NO_TRACE)
static __device__ long long g_trace_fused[4 * 8192];
#define FTRACE(i) do { if (threadIdx.x == 0 && blockIdx.x < 8192) g_trace_fused[4 * blockIdx.x + (i)] = wall_clock64(); } while (0)
#define FTRACE_G(gi) do { if (threadIdx.x == 0 && blockIdx.x < 8192) g_trace_fused[4 * blockIdx.x] = (wall_clock64() & ~7ll) | (gi); } while (0)
#define FTRACE_SET(i, v) do { if (threadIdx.x == 0 && blockIdx.x < 8192) g_trace_fused[4 * blockIdx.x + (i)] = (v); } while (0)
#define FTRACE_CLOCK() wall_clock64()
#define WGRAD_FUSED_TRACE_READER(name) \
    extern "C" int name(long long *host_out) { return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(::wgrad::g_trace_fused), sizeof(long long) * 4 * 8192); }
#else
#define FTRACE(i) do { } while (0)
#define FTRACE_G(gi) do { } while (0)
#define FTRACE_SET(i, v) do { (void)(v); } while (0)
#define FTRACE_CLOCK() 0ll
#define WGRAD_FUSED_TRACE_READER(name)
#endif

}  // namespace wgrad
