// bfloat16 storage elements: the upper half of an IEEE binary32 (1 sign bit, 8 exponent bits,
// 7 fraction bits).  Only the two conversions exist: the kernels widen every element as they
// read it and round the result once, to nearest with ties to even, as they store it.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace tcx {

struct bf16_t {
    unsigned short bits;

    bf16_t() = default;

    // float -> bfloat16: add half of the dropped field (one less when the kept field is even, so a
    // tie goes to the even neighbour) and cut.  The carry runs into the exponent as it should,
    // and up to the pattern of infinity on overflow.  NaNs keep their sign and turn quiet.
    static __device__ __forceinline__ unsigned short round_bits(uint32_t u) {
        if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x0040u);
        return (unsigned short)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    }
    __device__ __forceinline__ explicit bf16_t(float x) : bits(round_bits(__float_as_uint(x))) {}

    // double -> bfloat16 with ONE rounding: the double is first rounded to a float (24 bits);
    // only when that lands exactly on the midpoint of two bfloat16 values while the double was
    // not there can the second rounding go the wrong way, and then the float is nudged one
    // unit towards the side the double was on before it is rounded.
    __device__ __forceinline__ explicit bf16_t(double x) {
        const float f = (float)x;
        uint32_t u = __float_as_uint(f);
        if ((u & 0xffffu) == 0x8000u && (u & 0x7f800000u) != 0x7f800000u && (double)f != x)
            u = __builtin_fabs(x) > __builtin_fabs((double)f) ? u + 1u : u - 1u;
        bits = round_bits(u);
    }

    __device__ __forceinline__ explicit operator float() const { return __uint_as_float((uint32_t)bits << 16); }
    __device__ __forceinline__ explicit operator double() const { return (double)__uint_as_float((uint32_t)bits << 16); }
};
static_assert(sizeof(bf16_t) == 2, "storage element of 16 bits");

}  // namespace tcx
