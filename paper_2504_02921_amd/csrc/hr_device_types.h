// Device-side scalar helpers: storage types, conversions, wavefront (64-lane) reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hr_internal.h"

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
// Round to nearest even.  Nothing is clamped into the finite range: the bounds lie beyond the largest half (65504), so a
// magnitude the format cannot hold becomes infinity (and NaN becomes -infinity) and shows up as a non-finite score instead
// of a silently saturated one.  The min/max pair is kept for what it does to the instruction selection: without it a
// preceding multiplication is fused with the conversion into v_fma_mixlo_f16, which was measured to flush results below
// half's normal range (6.1e-5) to zero, and that is where the lo halves of split operands live (the all-layers-split test
// went from 1e-6 to 9e-5 against the float64 oracle).
template <> __device__ __forceinline__ half_t from_float<half_t>(float v) {
    return (half_t)fminf(fmaxf(v, -7.0e4f), 7.0e4f);
}

// A caller's value on its way to half: beyond the half range it becomes infinity; one that half cannot represent exactly
// (for a bf16 input: a magnitude below 2^-17, in half's subnormal range) is counted as inexact
__device__ __forceinline__ void count_half_range(float v, int& over, int& under, int& nonfinite) {
    const float a = fabsf(v);
    if (!(a <= 3.0e38f)) ++nonfinite;                 // NaN or infinity in the caller's data
    else if (a >= 65520.0f) ++over;
    else if ((float)(half_t)v != v) ++under;
}

// OCP E4M3 (bias 7, no infinities) decoded from its bit fields; exact in fp32.
__device__ __forceinline__ float e4m3_to_float(uint8_t c) {
    uint32_t sign = (uint32_t)(c & 0x80) << 24;
    uint32_t e = (c >> 3) & 0xF, m = c & 0x7;
    float mag = e == 0 ? (float)m * 0.001953125f : __uint_as_float(((e + 120u) << 23) | (m << 20));
    return __uint_as_float(__float_as_uint(mag) | sign);
}

// Rotate-half RoPE of one channel pair (x1 at index j, x2 at j + d/2) with explicit roundings, so that every kernel
// that applies it (the fused projection epilogue and the stand-alone RoPE kernels) produces the same bits.
__device__ __forceinline__ float rope_lo(float x1, float x2, float c, float s) { return __fmaf_rn(x1, c, -__fmul_rn(x2, s)); }
__device__ __forceinline__ float rope_hi(float x1, float x2, float c, float s) { return __fmaf_rn(x2, c, __fmul_rn(x1, s)); }

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
