// Element load / store helpers for the activation and output types.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace msgemm {

struct bf16_t { uint16_t bits; };  // bfloat16 storage

// b(.) of Section 3.1: two's-complement value of a 4-bit pattern.
__device__ __forceinline__ int decode4(unsigned nibble) { return (int)((nibble ^ 8u) & 15u) - 8; }

// Value of a 4-bit pattern for a table build: the plan's 16-entry value map for
// floating-point tables (the paper's b(.) unless the caller installed another
// encoding), b(.) itself for integer tables.
struct ValueMap { float v[16]; };  // travels by value in the launch arguments
__device__ __forceinline__ float code_value(const ValueMap& values, unsigned nibble, float) { return values.v[nibble & 15u]; }
__device__ __forceinline__ int code_value(const ValueMap&, unsigned nibble, int) { return decode4(nibble); }

template <typename T> struct XTraits;
template <> struct XTraits<float> {
    using acc_t = float;
    static __device__ __forceinline__ float load(const float* p) { return *p; }
};
template <> struct XTraits<__half> {
    using acc_t = float;
    static __device__ __forceinline__ float load(const __half* p) { return __half2float(*p); }
};
template <> struct XTraits<bf16_t> {
    using acc_t = float;
    static __device__ __forceinline__ float load(const bf16_t* p) {
        return __uint_as_float(((uint32_t)p->bits) << 16);
    }
};
template <> struct XTraits<int8_t> {
    using acc_t = int;
    static __device__ __forceinline__ int load(const int8_t* p) { return (int)*p; }
};

// Round-to-nearest-even conversions of an accumulator to the output type.
template <typename YT, typename AT> __device__ __forceinline__ YT to_output(AT v);
template <> __device__ __forceinline__ float to_output<float, float>(float v) { return v; }
template <> __device__ __forceinline__ __half to_output<__half, float>(float v) { return __float2half_rn(v); }
template <> __device__ __forceinline__ bf16_t to_output<bf16_t, float>(float v) {
    uint32_t u = __float_as_uint(v);
    bf16_t r;
    if ((u & 0x7fffffffu) > 0x7f800000u) {  // NaN stays NaN
        r.bits = (uint16_t)((u >> 16) | 0x0040u);
    } else {
        u += 0x7fffu + ((u >> 16) & 1u);
        r.bits = (uint16_t)(u >> 16);
    }
    return r;
}
template <> __device__ __forceinline__ int to_output<int, int>(int v) { return v; }

}  // namespace msgemm
