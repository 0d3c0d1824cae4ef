// Small device-side helpers shared by the kernel files (gfx950 only).
//
// The kernel files are compiled twice: once with brain-float as the 16-bit storage type (namespace ssk),
// once, with SS_HALF_F16 defined, with IEEE half (namespace ssk16).  Both formats are 16 bits wide, are
// multiplied by MFMA instructions of the same shape and rate and accumulate in fp32, so the kernels are the
// same text; what differs is collected here: the conversions, the element type of the MFMA operand
// vectors and the instruction names.  In the sources `bf16_t`, `bf2f`, `f2bf` and the BF16 dtype code
// therefore mean "the 16-bit type of this build".
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#ifdef SS_HALF_F16
#define SS_NS ssk16
#else
#define SS_NS ssk
#endif

namespace SS_NS {

typedef uint16_t bf16_t;   // raw bits of the 16-bit storage type

#ifdef SS_HALF_F16
typedef _Float16 half_elem_t;
#define SS_MFMA_32x32x16 __builtin_amdgcn_mfma_f32_32x32x16_f16
#define SS_MFMA_16x16x32 __builtin_amdgcn_mfma_f32_16x16x32_f16
#define SS_MFMA_16x16x32_ASM "v_mfma_f32_16x16x32_f16"
__device__ __forceinline__ float bf2f(bf16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }   // nearest even
#else
typedef __bf16 half_elem_t;
#define SS_MFMA_32x32x16 __builtin_amdgcn_mfma_f32_32x32x16_bf16
#define SS_MFMA_16x16x32 __builtin_amdgcn_mfma_f32_16x16x32_bf16
#define SS_MFMA_16x16x32_ASM "v_mfma_f32_16x16x32_bf16"
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ bf16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
#endif

// MFMA operand vector (8 elements) and packed pairs of the 16-bit type
typedef __attribute__((__vector_size__(8 * sizeof(half_elem_t)))) half_elem_t half8_t;
typedef float f32x2_cvt_t __attribute__((ext_vector_type(2)));
typedef half_elem_t half2_cvt_t __attribute__((ext_vector_type(2)));
// two floats -> packed pair, round to nearest even (one v_cvt_pk_* on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_cvt_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, half2_cvt_t));
}
// packed pair -> two floats
__device__ __forceinline__ void unpack_bf16x2(uint32_t w, float& lo, float& hi) {
#ifdef SS_HALF_F16
    lo = bf2f((bf16_t)(w & 0xffffu));
    hi = bf2f((bf16_t)(w >> 16));
#else
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xffff0000u);
#endif
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
    for (int i = 0; i < 4; ++i) unpack_bf16x2(v.w[i], f[2 * i], f[2 * i + 1]);
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
// In the rows of a V page whose head-dimension index e has bit 3 set, the two halves of the row are swapped on
// top of that: 16 lanes that read the same half of 16 consecutive rows (a fragment read of the second attention
// product out of LDS, where the page is kept as it is) then fall on 16 different bank groups instead of 8.
// vpos: position of token slot s in row e; vtok: token slot at position p of row e (its inverse).
__device__ __forceinline__ int vpos(int s, int e) { return vslot(s) ^ (e & 8); }
__device__ __forceinline__ int vtok(int p, int e) { return vslot(p ^ (e & 8)); }

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

}  // namespace SS_NS
