// Step 1 of Section 3.3 for one R block on bf16 MFMA, shared by the forward and the backward
// (which recomputes Y1): one wave computes D^T = R[kk] . X^T for 64 batch rows, all Q columns in
// accumulators.  The R fragments come packed in fragment order
//     RF1[kk][t][jt][lane][e] = R[kk][32*jt + lane%32][16*t + 8*(lane/32) + e]
// straight from global memory into a register ring three K-steps ahead (L2 latency); x arrives
// through a wave-private LDS ring of 64-column chunks filled by global_load_lds_dwordx4 in full
// 128-byte lines, two chunks ahead (HBM latency).
#pragma once
#include "monarch_mfma_common.h"

namespace monarch {

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt = simm16[3:0] | simm16[15:14] << 4)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// one global_load_lds_dwordx4: every lane fetches 16 bytes from its own address, the wave's 1 KiB
// lands contiguously at `lds_block` (+ lane * 16)
__device__ __forceinline__ void dma16(const uint16_t* gsrc, uint16_t* lds_block)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                     (__attribute__((address_space(3))) void*)lds_block, 16, 0, 0);
}

// 4 KiB staging unit = 32 rows x 128 bytes = four 1 KiB blocks of 8 rows.  One DMA instruction
// fills a block: lane s fetches row s/8, and its slot s%8 holds logical 16-byte piece
// (s%8) ^ key, key = (row & 7) ^ ((row >> 3) & 1), which makes the fragment reads conflict-free.
// The fragment for K-step u of the chunk (16 columns) is pieces 2u and 2u+1: lane (row = lane%32, g = lane/32).
__device__ __forceinline__ int unit_frag_off(int ln, int g, int u)
{
    const int bi = ln >> 3, r = ln & 7;
    return bi * 512 + r * 64 + 8 * ((2 * u + g) ^ r ^ (bi & 1));
}

// Compile-time shape of step 1: P inputs per block and the Q output columns one wave computes, N_IN = 4*P
// columns per row of x.  QTS: 32-wide j tiles per block in the packed R (more than QT when a block's
// columns are shared out over several waves); XRMAX: most ring slots a wave may use.
template <int P_, int Q_, int QTS_ = Q_ / 32, int XRMAX_ = 3>
struct Stage1 {
    static constexpr int P = P_, Q = Q_, N_IN = 4 * P_;
    static constexpr int NB = 2;              // two 32-row tiles
    static constexpr int QT = Q / 32;         // 32-wide j tiles of this wave
    static constexpr int QTS = QTS_;
    static constexpr int T1 = P / 16;         // K-steps
    static constexpr int C1 = P / 64;         // x chunks (64 columns = one 128-byte line per row)
    static constexpr int XR = C1 < XRMAX_ ? C1 : XRMAX_;  // x ring slots per wave (8 KiB each)
    static constexpr size_t LDS_X = (size_t)4 * XR * 8192;  // four waves
    // vmcnt values that guarantee an x chunk has landed: at most this many younger VMEM operations
    // may still be outstanding (stronger than necessary is safe, weaker is not)
    static constexpr int cap63(int v) { return v < 63 ? v : 63; }
    static constexpr int W_FIRST = cap63(8 * (XR - 1) + QT * (T1 < 3 ? T1 : 3));
    static constexpr int W_C0 = cap63(7 * QT + (XR > 2 ? 8 : 0));  // (+ the DMAs of chunk 2 when the prologue requested it)
    // (a ring of two slots: chunk c+1 was requested at the end of chunk c-1, only chunk c's R loads follow it)
    static constexpr int W_MID = XR == 2 ? cap63(4 * QT) : cap63(8 * QT + 8);
    static constexpr int W_LAST = XR == 2 ? cap63(4 * QT) : cap63(8 * QT);
    static_assert(P % 64 == 0 && Q % 32 == 0, "tile shapes");
};

// acc[jt*2 + nb] = D^T tile (j = (jt0 + jt)*32 .., b = nb*32 ..) of block kk for rows b0 .. b0+63 (rows past B
// are computed from row B-1 and must be dropped by the caller).  `ring` = this wave's XR * 8 KiB of LDS.
template <typename C>
__device__ __forceinline__ void stage1_block(const uint16_t* __restrict__ x, const uint16_t* __restrict__ RF1,
                                             int64_t b0, int64_t B, int kk, int lane, uint16_t* ring,
                                             f32x16 (&acc)[C::QT * C::NB], int jt0 = 0)
{
    const int ln = lane & 31, g = lane >> 5;
    const int rb = lane >> 3, pe = (lane & 7) ^ rb;
    const uint16_t* Xrow[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int64_t row = b0 + i * 8 + rb;
        row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
        Xrow[i] = x + row * C::N_IN + kk * C::P;
    }
    auto issue_x = [&](int c64) {
        uint16_t* dst = ring + (size_t)(c64 % C::XR) * 4096;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            dma16(Xrow[i] + c64 * 64 + 8 * (pe ^ (i & 1)), dst + i * 512);
    };
    int foff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) foff[u] = unit_frag_off(ln, g, u);
    // fragment (kk, t, jt): ((kk*T1 + t)*QTS + jt) * 512 elements, + lane * 8
    const uint16_t* Rk = RF1 + (((size_t)kk * C::T1 * C::QTS + jt0) * 64 + lane) * 8;

#pragma unroll
    for (int t = 0; t < C::QT * C::NB; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    u32x4 rf[4][C::QT], xf[2][C::NB];
    auto issue_r = [&](int t, int slot) {
#pragma unroll
        for (int jt = 0; jt < C::QT; ++jt) rf[slot][jt] = ldg128(Rk + (size_t)(t * C::QTS + jt) * 512);
    };
    auto read_x = [&](int c64, int u, int slot) {
        const uint16_t* buf = ring + (size_t)(c64 % C::XR) * 4096;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) xf[slot][nb] = lds128(buf + nb * 2048 + foff[u]);
    };
    // prologue: the first XR chunks of x, then the R fragments of K-steps 0..2
#pragma unroll
    for (int c = 0; c < C::XR; ++c) issue_x(c);
#pragma unroll
    for (int t = 0; t < 3; ++t)
        if (t < C::T1) issue_r(t, t);
    wait_vmcnt<C::W_FIRST>();
    __builtin_amdgcn_sched_barrier(0);
    read_x(0, 0, 0);

    for (int c64 = 0; c64 < C::C1; ++c64) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = c64 * 4 + u;
            __builtin_amdgcn_sched_barrier(0);
            if (t + 3 < C::T1) issue_r(t + 3, (u + 3) & 3);
            if (u < 3) {
                read_x(c64, u + 1, (u + 1) & 1);
            } else if (c64 + 1 < C::C1) {
                // chunk c64+1 has landed once only operations issued after its DMAs are outstanding
                if (c64 == 0) wait_vmcnt<C::W_C0>();
                else if (c64 + 2 < C::C1) wait_vmcnt<C::W_MID>();
                else wait_vmcnt<C::W_LAST>();
                __builtin_amdgcn_sched_barrier(0);
                read_x(c64 + 1, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int jt = 0; jt < C::QT; ++jt)
#pragma unroll
                for (int nb = 0; nb < C::NB; ++nb)
                    acc[jt * C::NB + nb] = mfma32(as_bf16x8(rf[u][jt]), as_bf16x8(xf[u & 1][nb]), acc[jt * C::NB + nb]);
            if (u == 3 && c64 + C::XR < C::C1) {
                __builtin_amdgcn_sched_barrier(0);
                wait_lgkmcnt0();  // the fragment reads of chunk c64 are done: its slot takes chunk c64+XR
                issue_x(c64 + C::XR);
            }
        }
    }
}

// The same product with two waves per block (eight waves per workgroup, two per SIMD, so that one wave's
// MFMAs run while the other waits for its loads): wave `half` of block kk computes the columns
// j in [half*Q/2, (half+1)*Q/2) -- acc[jl*2 + nb], jl = 0 .. QT/2-1 -- from its half of the R fragments,
// and both read x from one LDS ring (`ring` = the pair's XR * 8 KiB) that they fill together: each wave
// fetches its 32 rows of every chunk.  One workgroup barrier per chunk publishes the chunk and at the same
// time frees the slot of the chunk before it.  All eight waves of the workgroup must make the call.
template <typename C>
__device__ __forceinline__ void stage1_half(const uint16_t* __restrict__ x, const uint16_t* __restrict__ RF1,
                                            int64_t b0, int64_t B, int kk, int half, int lane, uint16_t* ring,
                                            f32x16 (&acc)[C::QT / 2 * C::NB])
{
    constexpr int QH = C::QT / 2, XR = 3;
    static_assert(C::QT % 2 == 0 && C::C1 >= XR, "column halves, ring depth");
    static_assert(8 * QH + 4 < 64, "vmcnt range");
    const int ln = lane & 31, g = lane >> 5;
    const int rb = lane >> 3, pe = (lane & 7) ^ rb;
    const uint16_t* Xrow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int64_t row = b0 + half * 32 + i * 8 + rb;
        row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
        Xrow[i] = x + row * C::N_IN + kk * C::P;
    }
    auto issue_x = [&](int c64) {  // this wave's 32 rows of chunk c64: four DMA instructions
        uint16_t* dst = ring + (size_t)(c64 % XR) * 4096 + half * 2048;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            dma16(Xrow[i] + c64 * 64 + 8 * (pe ^ (i & 1)), dst + i * 512);
    };
    int foff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) foff[u] = unit_frag_off(ln, g, u);
    const uint16_t* Rk = RF1 + (((size_t)kk * C::T1 * C::QT + half * QH) * 64 + lane) * 8;

#pragma unroll
    for (int t = 0; t < QH * C::NB; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    u32x4 rf[4][QH], xf[2][C::NB];
    auto issue_r = [&](int t, int slot) {
#pragma unroll
        for (int jl = 0; jl < QH; ++jl) rf[slot][jl] = ldg128(Rk + (size_t)(t * C::QT + jl) * 512);
    };
    auto read_x = [&](int c64, int u, int slot) {
        const uint16_t* buf = ring + (size_t)(c64 % XR) * 4096;
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) xf[slot][nb] = lds128(buf + nb * 2048 + foff[u]);
    };
    // prologue: chunks 0 and 1 of x, then the R fragments of K-steps 0..2.  Issue order after that, per
    // chunk c: [barrier] DMA of chunk c+2, then QH fragment loads in each of the chunk's four K-steps.
    issue_x(0);
    issue_x(1);
#pragma unroll
    for (int t = 0; t < 3; ++t) issue_r(t, t);

    for (int c64 = 0; c64 < C::C1; ++c64) {
        // this wave's part of chunk c64 has landed once only what was issued after it is outstanding:
        //   chunk 0: the DMA of chunk 1 and three K-steps of R;      chunk 1: 3 + 4 K-steps of R and the DMA of chunk 2;
        //   chunk c >= 2: the R loads of chunks c-2 and c-1 (eight K-steps) and the DMA of chunk c+1 (if there is one)
        if (c64 == 0) wait_vmcnt<4 + 3 * QH>();
        else if (c64 == 1) wait_vmcnt<7 * QH + (C::C1 > 2 ? 4 : 0)>();
        else if (c64 + 1 < C::C1) wait_vmcnt<8 * QH + 4>();
        else wait_vmcnt<8 * QH>();
        __builtin_amdgcn_sched_barrier(0);
        lds_barrier();  // the partner's rows are there too, and nobody reads chunk c64-1 any more (loads stay in flight)
        if (c64 + 2 < C::C1) issue_x(c64 + 2);
        read_x(c64, 0, 0);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = c64 * 4 + u;
            __builtin_amdgcn_sched_barrier(0);
            if (t + 3 < C::T1) issue_r(t + 3, (u + 3) & 3);
            if (u < 3) read_x(c64, u + 1, (u + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int jl = 0; jl < QH; ++jl)
#pragma unroll
                for (int nb = 0; nb < C::NB; ++nb)
                    acc[jl * C::NB + nb] = mfma32(as_bf16x8(rf[u][jl]), as_bf16x8(xf[u & 1][nb]), acc[jl * C::NB + nb]);
        }
    }
}

}  // namespace monarch
