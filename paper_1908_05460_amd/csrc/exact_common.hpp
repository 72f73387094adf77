// Pieces shared by the two exact-gradient kernels (gfx950).
#pragma once
#include "common.hpp"

namespace wgrad {

typedef float float4_t __attribute__((ext_vector_type(4)));

template <bool BF16>
__device__ __forceinline__ float load_elem(const void *p, long i)
{
    if (BF16) return bf16_bits_to_float(((const uint16_t *)p)[i]);
    return ((const float *)p)[i];
}

// V consecutive elements at a uniform base pointer plus a per-lane byte offset, widened to fp32 on use.
// settle(): passes the registers through opaque moves; placed after a load it puts the wait for that load
// there, and what follows sees registers with no load pending.
#define WGRAD_SETTLE(x) asm volatile("v_mov_b32 %0, %1" : "=v"(x) : "v"(x))
template <bool BF16, int V> struct Vec;
template <> struct Vec<false, 4> {
    float4_t r;
    __device__ __forceinline__ void load(const char *base, uint32_t off) { r = *(const float4_t *)(base + off); }
    __device__ __forceinline__ float get(int u) const { return r[u]; }
    __device__ __forceinline__ void settle() { float a = r[0], b = r[1], c = r[2], d = r[3]; WGRAD_SETTLE(a); WGRAD_SETTLE(b); WGRAD_SETTLE(c); WGRAD_SETTLE(d); r = float4_t{a, b, c, d}; }
};
template <> struct Vec<false, 2> {
    float2 r;
    __device__ __forceinline__ void load(const char *base, uint32_t off) { r = *(const float2 *)(base + off); }
    __device__ __forceinline__ float get(int u) const { return u == 0 ? r.x : r.y; }
    __device__ __forceinline__ void settle() { WGRAD_SETTLE(r.x); WGRAD_SETTLE(r.y); }
};
template <> struct Vec<true, 4> {
    uint2 r;
    __device__ __forceinline__ void load(const char *base, uint32_t off) { r = *(const uint2 *)(base + off); }
    __device__ __forceinline__ float get(int u) const {
        const uint32_t w = u < 2 ? r.x : r.y;
        return __uint_as_float((u & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    __device__ __forceinline__ void settle() { WGRAD_SETTLE(r.x); WGRAD_SETTLE(r.y); }
};
template <> struct Vec<true, 2> {
    uint32_t r;
    __device__ __forceinline__ void load(const char *base, uint32_t off) { r = *(const uint32_t *)(base + off); }
    __device__ __forceinline__ float get(int u) const { return __uint_as_float(u ? (r & 0xffff0000u) : (r << 16)); }
    __device__ __forceinline__ void settle() { WGRAD_SETTLE(r); }
};

}  // namespace wgrad
