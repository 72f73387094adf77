// Measured ceilings of the machine, for the benchmark only (built as libwgrad_roofs.so; nothing here is part
// of the library's C ABI or of the weight-gradient path).  Each kernel does one thing at the highest rate a
// plain HIP kernel reaches and the caller times it:
//   roof_copy        16-byte loads and stores, grid-stride             -> achievable HBM copy bandwidth
//   roof_read        16-byte loads only (the approximation streams dY) -> achievable HBM read bandwidth
//   roof_mfma_*      independent accumulators, no memory traffic       -> achievable matrix-core rate
//   roof_lds_read    conflict-free 4-byte LDS reads feeding one FMA each (the access pattern of the LDS-staged
//                    patch gather: one channel plane per lane, odd pitch)  -> achievable LDS read bandwidth
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void roof_copy(const uint4 *__restrict__ src, uint4 *__restrict__ dst, long n16)
{
    const long stride = (long)gridDim.x * 256;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void roof_read(const uint4 *__restrict__ src, uint32_t *__restrict__ sink, long n16)
{
    const long stride = (long)gridDim.x * 256;
    uint32_t acc = 0;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) {
        const uint4 v = src[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;          // never true for the benchmark's data; keeps the loads alive
}

// NACC independent accumulator tiles per wavefront, iters rounds over them.
template <int NACC>
__global__ __launch_bounds__(256) void roof_mfma_f32_16x16x4(float *__restrict__ sink, int iters)
{
    f32x4 acc[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float a = 1.0f + threadIdx.x * 1e-3f, b = 1.0f - threadIdx.x * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NACC; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (s == 12345.678f) sink[0] = s;
}

template <int NACC>
__global__ __launch_bounds__(256) void roof_mfma_bf16_16x16x32(float *__restrict__ sink, int iters)
{
    f32x4 acc[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(1.0f + 0.01f * i); b[i] = (__bf16)(1.0f - 0.01f * i); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NACC; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (s == 12345.678f) sink[0] = s;
}

template <int NACC>
__global__ __launch_bounds__(256) void roof_mfma_bf16_32x32x16(float *__restrict__ sink, int iters)
{
    f32x16 acc[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(1.0f + 0.01f * i); b[i] = (__bf16)(1.0f - 0.01f * i); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < NACC; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NACC; ++j) s += acc[j][0] + acc[j][5] + acc[j][10] + acc[j][15];
    if (s == 12345.678f) sink[0] = s;
}

// Every lane owns a plane of `pitch` floats (odd pitch: 32 consecutive lanes hit 32 banks) and reads a 3x3
// window of it per step, nine 4-byte reads each feeding one FMA, as the LDS-staged patch gather does.
__global__ __launch_bounds__(512) void roof_lds_read(float *__restrict__ sink, int iters, int pitch, int wp)
{
    extern __shared__ float xs[];
    const int tid = threadIdx.x, lane = tid & 63;
    for (int e = tid; e < 64 * pitch; e += 512) xs[e] = 1.0f + (e & 7);
    __syncthreads();
    const float *plane = xs + lane * pitch;
    float acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[t] = 0.f;
    int origin = (tid >> 6) & 3;
    for (int it = 0; it < iters; ++it) {
        const float *win = plane + origin;
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) acc[r * 3 + s] = fmaf(1.0001f, win[r * wp + s], acc[r * 3 + s]);
        origin = (origin + 1) & 3;                   // wavefront-uniform window origin, as in the gather
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 9; ++t) s += acc[t];
    if (s == 12345.678f) sink[0] = s;
}

extern "C" {

// Each call enqueues one launch on `stream` and returns hipGetLastError() as an int (0 = ok).
int roofs_copy(const void *src, void *dst, long bytes, void *stream)
{
    hipLaunchKernelGGL(roof_copy, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst, bytes / 16);
    return (int)hipGetLastError();
}

int roofs_read(const void *src, void *sink, long bytes, void *stream)
{
    hipLaunchKernelGGL(roof_read, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4 *)src, (uint32_t *)sink, bytes / 16);
    return (int)hipGetLastError();
}

// which: 0 = fp32 16x16x4, 1 = bf16 16x16x32, 2 = bf16 32x32x16.  blocks workgroups of 4 wavefronts, each wavefront
// issuing iters * nacc matrix instructions; *flops_out = the FLOPs of the whole launch.
int roofs_mfma(int which, int blocks, int iters, void *sink, double *flops_out, void *stream)
{
    const dim3 grid(blocks), block(256);
    hipStream_t st = (hipStream_t)stream;
    double per_instr = 0;
    int nacc = 0;
    if (which == 0)      { nacc = 16; per_instr = 2.0 * 16 * 16 * 4;  hipLaunchKernelGGL(roof_mfma_f32_16x16x4<16>, grid, block, 0, st, (float *)sink, iters); }
    else if (which == 1) { nacc = 16; per_instr = 2.0 * 16 * 16 * 32; hipLaunchKernelGGL(roof_mfma_bf16_16x16x32<16>, grid, block, 0, st, (float *)sink, iters); }
    else if (which == 2) { nacc = 4;  per_instr = 2.0 * 32 * 32 * 16; hipLaunchKernelGGL(roof_mfma_bf16_32x32x16<4>, grid, block, 0, st, (float *)sink, iters); }
    else return -1;
    if (flops_out) *flops_out = per_instr * nacc * (double)iters * 4.0 * blocks;
    return (int)hipGetLastError();
}

// blocks workgroups of 8 wavefronts; *bytes_out = LDS bytes read by the whole launch.
int roofs_lds_read(int blocks, int iters, void *sink, double *bytes_out, void *stream)
{
    const int wp = 10, pitch = 10 * 10 + 1;       // an 8x8 plane with its halo, odd pitch
    hipLaunchKernelGGL(roof_lds_read, dim3(blocks), dim3(512), 64 * pitch * sizeof(float), (hipStream_t)stream,
                       (float *)sink, iters, pitch, wp);
    if (bytes_out) *bytes_out = 9.0 * 4 * 512 * (double)iters * blocks;
    return (int)hipGetLastError();
}

}  // extern "C"
