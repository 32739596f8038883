// Output casts shared by the kernels of libepara: fp32 -> bf16 and fp32 -> OCP E4M3 ("fn": bias 7,
// 3 mantissa bits, no infinities, largest finite value 448), both round to nearest even.
#ifndef EPARA_CAST_H
#define EPARA_CAST_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace epara_cast {

// fp32 -> bf16 bits, round to nearest even.
__device__ __forceinline__ uint32_t f32_to_bf16(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// fp32 -> OCP E4M3 code, round to nearest even, saturating at +-448 (NaN -> 0x7f).
__device__ __forceinline__ uint32_t f32_to_e4m3(float x)
{
    const uint32_t u = __float_as_uint(x);
    const uint32_t sign = (u >> 24) & 0x80u;
    const uint32_t mag = u & 0x7fffffffu;
    if (mag > 0x7f800000u) return 0x7fu;
    const float a = __uint_as_float(mag);
    if (!(a < 448.f)) return sign | 0x7eu;
    if (a < 0.015625f)                                   // below 2^-6: multiples of 2^-9
        return sign | static_cast<uint32_t>(rintf(a * 512.f));
    uint32_t rnd = mag + 0x7ffffu + ((mag >> 20) & 1u);  // keep 3 mantissa bits
    uint32_t code = (rnd >> 20) - (120u << 3);           // rebias 127 -> 7
    return sign | (code > 0x7eu ? 0x7eu : code);
}

// Four fp32 values -> four E4M3 codes packed low byte first, round to nearest even, saturating at
// +-448 (v_cvt_pk_fp8_f32 after a clamp; gfx950 converts to the OCP format).  Finite inputs give the
// codes of f32_to_e4m3; a NaN input gives an unspecified code.
__device__ __forceinline__ uint32_t f32x4_to_e4m3(float a, float b, float c, float d)
{
    a = __builtin_amdgcn_fmed3f(a, -448.f, 448.f);
    b = __builtin_amdgcn_fmed3f(b, -448.f, 448.f);
    c = __builtin_amdgcn_fmed3f(c, -448.f, 448.f);
    d = __builtin_amdgcn_fmed3f(d, -448.f, 448.f);
    const int pk = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    return static_cast<uint32_t>(__builtin_amdgcn_cvt_pk_fp8_f32(c, d, pk, true));
}

}  // namespace epara_cast

#endif
