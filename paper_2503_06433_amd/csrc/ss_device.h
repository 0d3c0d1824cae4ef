// Small device-side helpers shared by the kernel files (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssk {

typedef uint16_t bf16_t;   // raw brain-float bits

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = f2bf(v); }

// 16-byte vector of raw storage
struct __attribute__((aligned(16))) vec16 { uint32_t w[4]; };

// streaming (touched once) 16-byte accesses: nontemporal hints keep them from displacing reusable lines
typedef uint32_t u32x4_nt __attribute__((ext_vector_type(4)));
__device__ __forceinline__ vec16 ld16_stream(const void* p) {
    const u32x4_nt v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(p));
    vec16 r;
    r.w[0] = v[0]; r.w[1] = v[1]; r.w[2] = v[2]; r.w[3] = v[3];
    return r;
}
__device__ __forceinline__ void st16_stream(void* p, const vec16& r) {
    const u32x4_nt v = {r.w[0], r.w[1], r.w[2], r.w[3]};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_nt*>(p));
}

template <typename T> struct VecOf;              // elements per 16 bytes
template <> struct VecOf<float> { static constexpr int N = 4; };
template <> struct VecOf<bf16_t> { static constexpr int N = 8; };

template <typename T> __device__ __forceinline__ void unpack16(const vec16& v, float* f);
template <> __device__ __forceinline__ void unpack16<float>(const vec16& v, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(v.w[i]);
}
template <> __device__ __forceinline__ void unpack16<bf16_t>(const vec16& v, float* f) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(v.w[i] << 16);
        f[2 * i + 1] = __uint_as_float(v.w[i] & 0xffff0000u);
    }
}
template <typename T> __device__ __forceinline__ vec16 pack16(const float* f);
template <> __device__ __forceinline__ vec16 pack16<float>(const float* f) {
    vec16 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v.w[i] = __float_as_uint(f[i]);
    return v;
}
template <> __device__ __forceinline__ vec16 pack16<bf16_t>(const float* f) {
    vec16 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v.w[i] = (uint32_t)f2bf(f[2 * i]) | ((uint32_t)f2bf(f[2 * i + 1]) << 16);
    return v;
}

// Position of token slot s (0..15) inside a 16-token row of a V page.  Rows keep the order
// [0-3, 8-11, 4-7, 12-15] (bits 2 and 3 of the slot swapped), so that the 8 tokens one MFMA lane
// group contributes to the second attention product are one contiguous 16-byte piece.
__device__ __forceinline__ int vslot(int s) { return (s & 3) | ((s & 4) << 1) | ((s & 8) >> 1); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

}  // namespace ssk
