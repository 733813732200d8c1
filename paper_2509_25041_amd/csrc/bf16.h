// bf16 <-> fp32 conversions (round-to-nearest-even on narrowing).  Pairs are narrowed with the
// packed hardware conversion of gfx950 (v_cvt_pk_bf16_f32), one instruction per two values.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace grace {

// 16-byte accesses that bypass cache retention (streamed rows are touched once)
typedef uint32_t u32x4_native __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 nt_load16(const uint4 *p) {
    const u32x4_native v = __builtin_nontemporal_load((const u32x4_native *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_store16(const uint4 &v, uint4 *p) {
    u32x4_native n;
    n.x = v.x; n.y = v.y; n.z = v.z; n.w = v.w;
    __builtin_nontemporal_store(n, (u32x4_native *)p);
}

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;  // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
typedef __bf16 bf16x2_native __attribute__((ext_vector_type(2)));
typedef float f32x2_native __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2_native v;
    v.x = lo;
    v.y = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_native));
}

__device__ __forceinline__ void unpack_bf16x8(const uint4 &v, float *f) {
    f[0] = bf16_lo_to_f32(v.x); f[1] = bf16_hi_to_f32(v.x);
    f[2] = bf16_lo_to_f32(v.y); f[3] = bf16_hi_to_f32(v.y);
    f[4] = bf16_lo_to_f32(v.z); f[5] = bf16_hi_to_f32(v.z);
    f[6] = bf16_lo_to_f32(v.w); f[7] = bf16_hi_to_f32(v.w);
}
__device__ __forceinline__ uint4 pack_bf16x8(const float *f) {
    uint4 o;
    o.x = pack_bf16x2(f[0], f[1]); o.y = pack_bf16x2(f[2], f[3]);
    o.z = pack_bf16x2(f[4], f[5]); o.w = pack_bf16x2(f[6], f[7]);
    return o;
}
__device__ __forceinline__ void unpack_f32x4(const uint4 &v, float *f) {
    f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
    f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
}
__device__ __forceinline__ uint4 pack_f32x4(const float *f) {
    uint4 o;
    o.x = __float_as_uint(f[0]); o.y = __float_as_uint(f[1]);
    o.z = __float_as_uint(f[2]); o.w = __float_as_uint(f[3]);
    return o;
}

}  // namespace grace
