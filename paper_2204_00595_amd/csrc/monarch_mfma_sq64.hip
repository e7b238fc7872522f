// bf16 kernels for the square Monarch matrix of Definition 3.1 with m = 64 (n = 4096,
// k = q = s = p = 64): fused forward here, backward data path in `bwd_sq64_data_kernel`.
//
// Per batch row the input is a 64 x 64 matrix X[kk][i].  Step 1 of Section 3.3 multiplies
// row kk by R[kk], the permutation turns the result Y1[kk][j] into U[c][r] = Y1[r][c], step 2
// multiplies row c of U (column c of Y1) by L[c], and step 3 writes y[l*64 + c] = W[c][l].  So
// every output block needs one column from every input block: a workgroup has to own whole rows,
// 8 KiB each in bf16.  A workgroup (8 waves) owns 32 rows; wave w computes blocks kk = 8w..8w+7 of
// step 1 and keeps the 32 x 512 results packed in registers (pairs of kk per dword), because the
// full 256 KiB intermediate does not fit in LDS.  It is exchanged in two halves (columns
// j < 32, then j >= 32): each half is written to LDS as U[b][j][kk] (kk fastest, 16-byte writes
// of the wave's eight kk), which is exactly the operand order of step 2 for block c = j, and step 2
// for the 32 blocks of that half runs before the other half is exchanged.
//
// MFMA operands are loaded from global memory in operand layout.  Which contraction index sits
// in which K-slot is free as long as both operands agree, so lane group g of K-step u takes
// i = 32g + 8u .. +7: every lane then reads 64 contiguous bytes of its row.
// Step-2 results of eight consecutive c are packed per lane, so that y is written in 16-byte
// pieces y[b][l*64 + c0 .. c0+7].
#include "monarch_internal.h"
#include "monarch_mfma_common.h"
#include <cstdlib>

namespace monarch {

namespace {

constexpr int M64 = 64, N64 = 4096;
constexpr int SQ_BM = 32;                          // rows per workgroup
constexpr int SQ_ROWB = 32 * 128 + 16;             // bytes per row of the exchange buffer (32 j x 64 kk + pad)
constexpr size_t SQ_LDS = (size_t)SQ_BM * SQ_ROWB; // 131584 bytes

template <int DBG>
__global__ void __launch_bounds__(512)
fwd_sq64_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ R,
                const uint16_t* __restrict__ L, uint16_t* __restrict__ y, int64_t B)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ldsb[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 31, g = lane >> 5;
    const int64_t b0 = (int64_t)blockIdx.x * SQ_BM;
    int64_t row = b0 + ln;
    const bool row_ok = row < B;
    row = row_ok ? row : B - 1;  // rows past the end are computed from a valid row and dropped

    // ---------------------------------------------------------------- step 1 ----
    // Results as bf16 pairs (kk even, kk odd) of Y1[b = ln][kk][j], j = 32*jt + 8*(i/4) + 4*g + i%4.
    // The half j < 32 goes to the exchange buffer as it is produced (LDS is idle during step 1),
    // the half j >= 32 stays in pk1[t2][i] until the first half has been consumed.
    uint32_t pk1[4][16];
    {
        const uint16_t* xrow = x + row * N64 + (size_t)wave * 8 * M64 + 32 * g;
        const uint16_t* Rrow = R + ((size_t)wave * 8 * M64 + ln) * M64 + 32 * g;
        u32x4 xa[2][4], ra[2][4];
        auto load_x = [&](int t, int s) {
#pragma unroll
            for (int u = 0; u < 4; ++u) xa[s][u] = DBG == 4 ? u32x4{(uint32_t)t, 1u, 2u, 3u} : ldg128(xrow + t * M64 + 8 * u);
        };
        auto load_r = [&](int t, int jt) {
#pragma unroll
            for (int u = 0; u < 4; ++u) ra[jt][u] = DBG == 2 ? u32x4{(uint32_t)t, 1u, 2u, 3u} : ldg128(Rrow + ((size_t)t * M64 + 32 * jt) * M64 + 8 * u);
        };
        load_x(0, 0);
        load_r(0, 0);
        load_r(0, 1);
        f32x16 ev[2];
        uint32_t q0[2][16];
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int s = t & 1;
            __builtin_amdgcn_sched_barrier(0);  // pins the prefetch distance
            if (t + 1 < 8) load_x(t + 1, s ^ 1);
#pragma unroll
            for (int jt = 0; jt < 2; ++jt) {
                __builtin_amdgcn_sched_barrier(0);
                f32x16 acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
                for (int u = 0; u < 4; ++u) acc = mfma32(as_bf16x8(ra[jt][u]), as_bf16x8(xa[s][u]), acc);
                __builtin_amdgcn_sched_barrier(0);
                if (t + 1 < 8) load_r(t + 1, jt);
                if ((t & 1) == 0) {
                    ev[jt] = acc;
                } else if (jt == 1) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) pk1[t >> 1][i] = pack_bf16x2(ev[1][i], acc[i]);
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) q0[(t >> 1) & 1][i] = pack_bf16x2(ev[0][i], acc[i]);
                    if ((t & 3) == 3) {
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const int jl = 8 * (i >> 2) + 4 * g + (i & 3);
                            *reinterpret_cast<u32x2*>(ldsb + (size_t)ln * SQ_ROWB + jl * 128 + 16 * wave + 8 * (t >> 2)) =
                                u32x2{q0[0][i], q0[1][i]};
                        }
                    }
                }
            }
        }
    }

    // ------------------------------------------------- exchange + step 2, two halves ----
    // po[h][c2][i]: bf16 pair (c0 + 2*c2, c0 + 2*c2 + 1) of W[b = ln][c][l], c0 = 32h + 8cg,
    // l = 32*lt + 8*(i/4) + 4*g + i%4
    const int cg = wave & 3, lt = wave >> 2;  // eight blocks c of the half, one 32-row tile of l
    uint32_t po[2][4][16];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (h) {
            __syncthreads();  // step 2 of the first half has read everything it needs
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int jl = 8 * (i >> 2) + 4 * g + (i & 3);
                *reinterpret_cast<u32x4*>(ldsb + (size_t)ln * SQ_ROWB + jl * 128 + 16 * wave) =
                    u32x4{pk1[0][i], pk1[1][i], pk1[2][i], pk1[3][i]};
            }
        }
        __syncthreads();

        const unsigned char* ub = ldsb + (size_t)ln * SQ_ROWB + (8 * cg) * 128 + 64 * g;
        const uint16_t* Lrow = L + (((size_t)(32 * h + 8 * cg)) * M64 + 32 * lt + ln) * M64 + 32 * g;
        u32x4 la[2][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) la[0][u] = ldg128(Lrow + 8 * u);
        f32x16 ev;
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
            const int s = cc & 1;
            __builtin_amdgcn_sched_barrier(0);
            if (cc + 1 < 8) {
#pragma unroll
                for (int u = 0; u < 4; ++u) la[s ^ 1][u] = DBG == 3 ? u32x4{(uint32_t)cc, 1u, 2u, 3u} : ldg128(Lrow + (size_t)(cc + 1) * M64 * M64 + 8 * u);
            }
            __builtin_amdgcn_sched_barrier(0);
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const u32x4 ua = *reinterpret_cast<const u32x4*>(ub + cc * 128 + 16 * u);
                acc = mfma32(as_bf16x8(la[s][u]), as_bf16x8(ua), acc);
            }
            if ((cc & 1) == 0) {
                ev = acc;
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) po[h][cc >> 1][i] = pack_bf16x2(ev[i], acc[i]);
            }
        }
    }

    // ---------------------------------------------------------------- step 3 ----
    // y[b][l*64 + c] is written in full 128-byte lines (all 64 c of one (b, l)): the results are
    // transposed through LDS, one 32-row tile of l per round.  LDS tile: [b][l][8 pieces of 16 B],
    // piece index XOR-ed with b % 8 so that the writes of 8 adjacent lanes hit 8 different slots.
#pragma unroll
    for (int rnd = 0; rnd < 2; ++rnd) {
        __syncthreads();  // the exchange buffer (or the previous round's tile) is dead
        if (lt == rnd) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int l = 8 * (i >> 2) + 4 * g + (i & 3);
                    const int piece = (4 * h + cg) ^ (ln & 7);
                    *reinterpret_cast<u32x4*>(ldsb + (size_t)ln * 4096 + l * 128 + piece * 16) =
                        u32x4{po[h][0][i], po[h][1][i], po[h][2][i], po[h][3][i]};
                }
        }
        __syncthreads();
        // wave w copies rows b = 4w .. 4w+3: 128 lines, eight per instruction (1 KiB contiguous in y)
#pragma unroll
        for (int k2 = 0; k2 < 16; ++k2) {
            const int line = 8 * k2 + (lane >> 3), pc = lane & 7;
            const int b = 4 * wave + (line >> 5), l = line & 31;
            const u32x4 v = *reinterpret_cast<const u32x4*>(ldsb + (size_t)b * 4096 + l * 128 + ((pc ^ (b & 7)) * 16));
            if (DBG != 1 && b0 + b < B)
                *reinterpret_cast<u32x4*>(y + (b0 + b) * N64 + (size_t)(32 * rnd + l) * M64 + 8 * pc) = v;
        }
    }
}

}  // namespace

bool sq64_supported(const Problem& pb)
{
    return pb.dtype == 1 && pb.k == 64 && pb.p == 64 && pb.q == 64 && pb.s == 64;
}

int fwd_sq64(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if (!sq64_supported(pb)) return -2;
    static const int v = getenv("MONARCH_SQ64_VARIANT") ? atoi(getenv("MONARCH_SQ64_VARIANT")) : 0;  // TUNING
    auto kern = v == 1 ? fwd_sq64_kernel<1> : v == 2 ? fwd_sq64_kernel<2> : v == 3 ? fwd_sq64_kernel<3> : v == 4 ? fwd_sq64_kernel<4> : fwd_sq64_kernel<0>;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SQ_LDS) != hipSuccess)
        return -4;
    const int64_t grid = (pb.B + SQ_BM - 1) / SQ_BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ_LDS, st, (const uint16_t*)x, (const uint16_t*)R,
                       (const uint16_t*)L, (uint16_t*)y, pb.B);
    return hip_status(hipGetLastError());
}

}  // namespace monarch
