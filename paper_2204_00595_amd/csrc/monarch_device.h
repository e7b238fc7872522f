// Device-side helpers shared by the kernel families.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace monarch {

typedef uint16_t bf16_t;  // storage type: upper half of a binary32

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// Round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Position g in U (the stage-2 input vector, length k*q) that receives stage-1 output
// f = kk*q + j.  Default reading: U[g] = Y1[g mod k][g div k]  =>  g = j*k + kk.
// Alternative reading:            U[c*q + r] = Y1flat[r*k + c]   =>  g = (f mod k)*q + f div k.
__device__ __forceinline__ int mid_dest(int f, int k, int q, bool perm_b)
{
    if (!perm_b) { int kk = f / q, j = f - kk * q; return j * k + kk; }
    int r = f / k, c = f - r * k;
    return c * q + r;
}

}  // namespace monarch
