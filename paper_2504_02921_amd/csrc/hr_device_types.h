// Device-side scalar helpers: storage types, conversions, wavefront (64-lane) reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hr {

typedef __bf16 bf16_t;      // storage type of the caller's 16-bit weights, embedding and KV
typedef _Float16 half_t;    // the library's 16-bit compute / activation type (MFMA operand type)

template <typename T> __device__ __forceinline__ float to_float(T v);
template <> __device__ __forceinline__ float to_float<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_float<bf16_t>(bf16_t v) { return (float)v; }
template <> __device__ __forceinline__ float to_float<half_t>(half_t v) { return (float)v; }

template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return (bf16_t)v; }   // round to nearest even
// round to nearest even, saturating at the largest finite half instead of overflowing to infinity
template <> __device__ __forceinline__ half_t from_float<half_t>(float v) {
    return (half_t)fminf(fmaxf(v, -65504.0f), 65504.0f);
}

// OCP E4M3 (bias 7, no infinities) decoded from its bit fields; exact in fp32.
__device__ __forceinline__ float e4m3_to_float(uint8_t c) {
    uint32_t sign = (uint32_t)(c & 0x80) << 24;
    uint32_t e = (c >> 3) & 0xF, m = c & 0x7;
    float mag = e == 0 ? (float)m * 0.001953125f : __uint_as_float(((e + 120u) << 23) | (m << 20));
    return __uint_as_float(__float_as_uint(mag) | sign);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

}  // namespace hr
