// Device-side element helpers: storage types and conversions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ms {

// bfloat16 storage: the upper 16 bits of an IEEE-754 binary32.
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits) { return __uint_as_float(bits << 16); }

// Round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Sum over a workgroup of kThreads threads; every thread gets the total.  red: kThreads / 64 floats of LDS.
template <int kThreads>
__device__ __forceinline__ float block_sum(float x, float* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = x;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < kThreads / 64; ++i) t += red[i];
    return t;
}

// Row kernels with a norm (one workgroup per row, the row held in registers between the two passes):
// threads per row and 8-element chunks per thread; rows of up to 8192 elements.
constexpr int kNormThreads = 512;
constexpr int kNormMaxPerThread = 2;

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return bf16_bits_to_float(x.bits); }

template <typename T>
__device__ __forceinline__ T from_float(float f);
template <>
__device__ __forceinline__ float from_float<float>(float f) {
    return f;
}
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float f) {
    bf16_t r;
    r.bits = float_to_bf16_bits(f);
    return r;
}

}  // namespace ms
