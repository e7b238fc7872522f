// MFMA helpers for gfx950 (CDNA4): operand types, fragment loads, bf16 packing.
//
// Register layouts used throughout (64-lane wavefront, lane = threadIdx.x % 64):
//   v_mfma_f32_32x32x16_bf16   A (32 x 16): lane holds row  lane%32, K-slots 8*(lane/32) .. +7
//                              B (16 x 32): lane holds col  lane%32, K-slots 8*(lane/32) .. +7
//                              D (32 x 32): acc[i] = D[8*(i/4) + 4*(lane/32) + i%4][lane%32]
//   v_mfma_f32_16x16x32_bf16   A (16 x 32): row lane%16, K-slots 8*(lane/16) .. +7;  B likewise
//                              D (16 x 16): acc[i] = D[4*(lane/16) + i][lane%16]
//   v_mfma_f32_16x16x4_f32     A (16 x 4):  row lane%16, K-slot lane/16;             B likewise
//                              D (16 x 16): acc[i] = D[4*(lane/16) + i][lane%16]
// Which contraction index sits in which K-slot is free as long as A and B agree; the
// kernels use that freedom to fold the Monarch permutations into the operand loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace monarch {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// two floats -> two bf16 (round to nearest even) packed in one dword, `lo` in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 f = {lo, hi};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ u32x4 ldg128(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
// streaming (non-temporal) 16-byte global accesses for data touched once per launch
__device__ __forceinline__ u32x4 ldg128_nt(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)); }
__device__ __forceinline__ void stg128_nt(void* p, u32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p)); }
__device__ __forceinline__ f32x4 ldg128f_nt(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p)); }
__device__ __forceinline__ void stg128f_nt(void* p, f32x4 v) { __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p)); }
__device__ __forceinline__ u32x4 lds128(const void* p) { return *reinterpret_cast<const u32x4*>(p); }

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// Workgroup barrier for data handed over through LDS, which leaves global loads in flight.
// __syncthreads() carries workgroup-scope fences, for which the compiler makes the wave wait until every
// outstanding global load has returned (s_waitcnt vmcnt(0)) -- a fence restricted to LDS does the same for
// global_load_lds requests, which count as LDS writes.  A prefetch that is meant to stay in flight across the
// barrier is drained there, and the wave pays the full memory latency at every barrier.  Here the wave waits
// for its own LDS operations only (lgkmcnt(0)); the empty asm statements keep the compiler from moving memory
// operations across.  What global_load_lds (DMA) writes into LDS is NOT covered: the wave that requested it
// waits for it explicitly (s_waitcnt vmcnt(n)) before it arrives here.  Keep __syncthreads() wherever global
// memory written by one wave is read by another after the barrier.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// (lo16 of a) | (lo16 of b) << 16   and   (hi16 of a) | (hi16 of b) << 16
__device__ __forceinline__ uint32_t pick_lo16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pick_hi16(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

}  // namespace monarch
