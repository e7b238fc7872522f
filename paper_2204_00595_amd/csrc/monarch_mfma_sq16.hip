// fp32 kernels for the square Monarch matrix of Definition 3.1 with m = 16 (n = 256,
// k = q = s = p = 16) on v_mfma_f32_16x16x4_f32.
//
// This shape moves 2 KiB per batch row for 16 KFLOP: it is bound by HBM bandwidth (or, for a
// few rows, by launch latency).  The design therefore keeps the weights on chip for the whole
// launch and touches every activation byte once, in full cache lines:
//   * persistent workgroups of 8 waves; R and L (16 KiB each) are loaded once into LDS in MFMA
//     operand order (one 16-byte read per block and lane);
//   * a wave owns 16 batch rows at a time.  Step 1 of Section 3.3 for block kk is
//     D[j][b] = sum_i R[kk][j][i] x[b][16kk + i]: four K = 4 MFMAs whose x operand is one 16-byte
//     load per lane (K-slot h of MFMA u takes i = 4h + u; the slot assignment is free as long as
//     both operands agree);
//   * the permutation P^T (U[c][r] = Y1[r][c]) is a pass through a wave-private 16 KiB LDS tile
//     T[b][kk][j]: written as produced (16-byte pieces), read back as the step-2 operand
//     T[b][4h + u][0..15];
//   * step 2 leaves lane (b, h) with the 64 consecutive outputs y[b][64h .. 64h + 63] (step 3
//     needs no data movement); they take one more pass through the tile so that every store
//     instruction writes one full 1 KiB row.
// No workgroup barrier after the weights are in LDS: waves run independently.
#include "monarch_internal.h"
#include "monarch_mfma_common.h"

namespace monarch {

namespace {

constexpr int N16 = 256;
constexpr int SQ16_WAVES = 8;
constexpr size_t SQ16_W_BYTES = 16 * 64 * 16;                      // one factor in operand order
constexpr size_t SQ16_T_BYTES = 16 * 1024;                         // one wave's tile
constexpr size_t SQ16_LDS = 2 * SQ16_W_BYTES + SQ16_WAVES * SQ16_T_BYTES;  // 160 KiB

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// orders LDS traffic of one wave: what lanes wrote before is visible to the reads after
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// tile T: 16 rows of 64 16-byte pieces; piece index XOR-ed with row % 8 (bank spreading)
__device__ __forceinline__ int t_off(int row, int piece) { return row * 1024 + ((piece ^ (row & 7)) << 4); }

// W[block][row][col] (fp32, 16 x 16 x 16) -> LDS operand order: dst[block][lane] = W[block][lane % 16][4 * (lane / 16) .. +3]
__device__ __forceinline__ void stage_weights(const float* __restrict__ W, unsigned char* dst, int tid, int nthreads)
{
    for (int e = tid; e < 16 * 64; e += nthreads) {
        const int blk = e >> 6, lane = e & 63;
        *reinterpret_cast<f32x4*>(dst + (size_t)e * 16) =
            *reinterpret_cast<const f32x4*>(W + ((size_t)blk * 16 + (lane & 15)) * 16 + 4 * (lane >> 4));
    }
}

__global__ void __launch_bounds__(512)
fwd_sq16_kernel(const float* __restrict__ x, const float* __restrict__ R, const float* __restrict__ L,
                float* __restrict__ y, int64_t B, int64_t ntiles)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ldsb[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int bl = lane & 15, h = lane >> 4;
    unsigned char* Rop = ldsb;
    unsigned char* Lop = ldsb + SQ16_W_BYTES;
    unsigned char* T = ldsb + 2 * SQ16_W_BYTES + (size_t)wave * SQ16_T_BYTES;
    stage_weights(R, Rop, tid, 512);
    stage_weights(L, Lop, tid, 512);
    __syncthreads();

    const int64_t stride = (int64_t)gridDim.x * SQ16_WAVES;
    int64_t tile = (int64_t)blockIdx.x * SQ16_WAVES + wave;
    auto load_x = [&](int64_t tl, f32x4 (&xa)[16]) {
        int64_t row = tl * 16 + bl;
        row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
        const float* p = x + row * N16 + 4 * h;
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) xa[kk] = *reinterpret_cast<const f32x4*>(p + 16 * kk);
    };
    f32x4 xa[16];
    if (tile < ntiles) load_x(tile, xa);
    for (; tile < ntiles; tile += stride) {
        // ---- step 1: Y1[b][kk][j = 4h + i] -> T[b][kk][j]
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const f32x4 ra = *reinterpret_cast<const f32x4*>(Rop + ((size_t)kk * 64 + lane) * 16);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma4(ra[u], xa[kk][u], acc);
            *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * kk + h)) = acc;
        }
        // the next tile's rows are fetched while this one is finished
        const int64_t next = tile + stride;
        if (next < ntiles) load_x(next, xa);
        wave_lds_fence();
        // ---- step 2 operand: ub[u][c] = U[b][c][r = 4h + u] = Y1[b][kk = 4h + u][j = c]
        f32x4 ub[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) ub[u][v] = *reinterpret_cast<const f32x4*>(T + t_off(bl, 4 * (4 * h + u) + v));
        // ---- step 2: W[b][c][l = 4h + i]; y[b][16 l + c]: lane (b, h) owns y[b][64h + 16 i + c]
        f32x4 w[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const f32x4 la = *reinterpret_cast<const f32x4*>(Lop + ((size_t)c * 64 + lane) * 16);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma4(la[u], ub[u][c >> 2][c & 3], acc);
            w[c] = acc;
        }
        wave_lds_fence();  // every lane has read its operands: the tile is reused for y
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int cq = 0; cq < 4; ++cq)
                *reinterpret_cast<f32x4*>(T + t_off(bl, 16 * h + 4 * i + cq)) =
                    f32x4{w[4 * cq][i], w[4 * cq + 1][i], w[4 * cq + 2][i], w[4 * cq + 3][i]};
        wave_lds_fence();
        // ---- step 3: one full row (1 KiB) per store instruction
        const int64_t b0 = tile * 16;
#pragma unroll
        for (int k2 = 0; k2 < 16; ++k2) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(T + t_off(k2, lane));
            if (b0 + k2 < B) *reinterpret_cast<f32x4*>(y + (b0 + k2) * N16 + 4 * lane) = v;
        }
        wave_lds_fence();  // the tile is free again for the next step 1
    }
}

}  // namespace

bool sq16_supported(const Problem& pb)
{
    // both readings of the mid permutation coincide when k = q
    return pb.dtype == 0 && pb.k == 16 && pb.p == 16 && pb.q == 16 && pb.s == 16;
}

int fwd_sq16(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if (!sq16_supported(pb)) return -2;
    auto kern = fwd_sq16_kernel;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)SQ16_LDS) != hipSuccess)
        return -4;
    const int64_t ntiles = (pb.B + 15) / 16;
    int64_t grid = (ntiles + SQ16_WAVES - 1) / SQ16_WAVES;
    if (grid > 256) grid = 256;  // one persistent workgroup per CU
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ16_LDS, st, (const float*)x, (const float*)R,
                       (const float*)L, (float*)y, pb.B, ntiles);
    return hip_status(hipGetLastError());
}

}  // namespace monarch
