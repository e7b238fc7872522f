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

// W[block][row][col] (fp32, 16 x 16 x 16) -> LDS operand order: dst[block][lane] = W[block][lane % 16][4 * (lane / 16) .. +3].
// NT threads take 1024 / NT pieces each; all of a thread's loads are issued before its first LDS store, so the
// staging costs one memory latency (a launch with a handful of tiles is mostly this latency).
template <int NT>
__device__ __forceinline__ void stage_weights(const float* __restrict__ W, unsigned char* dst, int tid)
{
    constexpr int PER = 16 * 64 / NT;
    f32x4 v[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int e = tid + k * NT, blk = e >> 6, lane = e & 63;
        v[k] = *reinterpret_cast<const f32x4*>(W + ((size_t)blk * 16 + (lane & 15)) * 16 + 4 * (lane >> 4));
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) *reinterpret_cast<f32x4*>(dst + (size_t)(tid + k * NT) * 16) = v[k];
}

template <bool BIAS>
__global__ void __launch_bounds__(512)
fwd_sq16_kernel(const float* __restrict__ x, const float* __restrict__ R, const float* __restrict__ L,
                const float* __restrict__ bias, float* __restrict__ y, int64_t B, int64_t ntiles)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ldsb[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int bl = lane & 15, h = lane >> 4;
    unsigned char* Rop = ldsb;
    unsigned char* Lop = ldsb + SQ16_W_BYTES;
    unsigned char* T = ldsb + 2 * SQ16_W_BYTES + (size_t)wave * SQ16_T_BYTES;
    const int64_t stride = (int64_t)gridDim.x * SQ16_WAVES;
    int64_t tile = (int64_t)blockIdx.x * SQ16_WAVES + wave;
    auto load_x = [&](int64_t tl, f32x4 (&xa)[16]) {
        int64_t row = tl * 16 + bl;
        row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
        const float* p = x + row * N16 + 4 * h;
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) xa[kk] = ldg128f_nt(p + 16 * kk);
    };
    f32x4 xa[16];
    if (tile < ntiles) load_x(tile, xa);  // in flight while the weights are staged
    f32x4 bv = {0.f, 0.f, 0.f, 0.f};  // the lane stores y[b][4*lane .. 4*lane + 3] of every row
    if constexpr (BIAS) bv = *reinterpret_cast<const f32x4*>(bias + 4 * lane);
    stage_weights<512>(R, Rop, tid);
    stage_weights<512>(L, Lop, tid);
    __syncthreads();
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
            f32x4 v = *reinterpret_cast<const f32x4*>(T + t_off(k2, lane));
            if constexpr (BIAS) v += bv;
            if (b0 + k2 < B) stg128f_nt(y + (b0 + k2) * N16 + 4 * lane, v);
        }
        wave_lds_fence();  // the tile is free again for the next step 1
    }
}

// Short batches (up to 2048 tiles): one four-wave workgroup per 16-row tile.  The persistent kernel above pays, per
// launch, for staging both factors into LDS behind a workgroup barrier, which is the price of a launch that has many
// more tiles than waves; here wave q takes the blocks kk = 4q .. 4q+3 of step 1 and c = 4q .. 4q+3 of step 2 and reads
// their operands of R and L (the same operand order) straight from global memory while its rows of x are in flight:
// twelve loads and 32 MFMAs per wave, three workgroup barriers around the 16 KiB tile.  The latency of a short batch is
// one tile's chain of loads, MFMAs and exchanges, which the split shortens (64 rows: 5.0 -> 3.2 us against one wave per tile).
template <bool BIAS>
__global__ void __launch_bounds__(256)
fwd_sq16_tile_kernel(const float* __restrict__ x, const float* __restrict__ R, const float* __restrict__ L,
                     const float* __restrict__ bias, float* __restrict__ y, int64_t B)
{
    __shared__ __attribute__((aligned(16))) unsigned char T[SQ16_T_BYTES];
    const int tid = threadIdx.x, lane = tid & 63;
    const int q = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bl = lane & 15, h = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * 16;
    int64_t row = b0 + bl;
    row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
    f32x4 xa[4], ra[4], la[4];
    const float* px = x + row * N16 + 4 * h;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int blk = 4 * q + w;
        xa[w] = ldg128f_nt(px + 16 * blk);
        ra[w] = *reinterpret_cast<const f32x4*>(R + ((size_t)blk * 16 + bl) * 16 + 4 * h);
        la[w] = *reinterpret_cast<const f32x4*>(L + ((size_t)blk * 16 + bl) * 16 + 4 * h);
    }
    f32x4 bv = {0.f, 0.f, 0.f, 0.f};
    if constexpr (BIAS) bv = *reinterpret_cast<const f32x4*>(bias + 4 * lane);
    __builtin_amdgcn_sched_barrier(0);  // every load is issued before the first use
    // ---- step 1: Y1[b][kk][j = 4h + i] -> T[b][kk][j], kk = 4q + w
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = mfma4(ra[w][u], xa[w][u], acc);
        *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * (4 * q + w) + h)) = acc;
    }
    __syncthreads();
    // ---- step 2 operand: ub[u] = U[b][c = 4q .. 4q+3][r = 4h + u] = Y1[b][kk = 4h + u][j = c]
    f32x4 ub[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) ub[u] = *reinterpret_cast<const f32x4*>(T + t_off(bl, 4 * (4 * h + u) + q));
    f32x4 wv[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = mfma4(la[w][u], ub[u][w], acc);
        wv[w] = acc;
    }
    __syncthreads();  // every wave has read its operands: the tile is reused for y
#pragma unroll
    for (int i = 0; i < 4; ++i)
        *reinterpret_cast<f32x4*>(T + t_off(bl, 16 * h + 4 * i + q)) = f32x4{wv[0][i], wv[1][i], wv[2][i], wv[3][i]};
    __syncthreads();
    // ---- step 3: one full row (1 KiB) per store instruction, four rows per wave
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int k2 = 4 * q + w;
        f32x4 v = *reinterpret_cast<const f32x4*>(T + t_off(k2, lane));
        if constexpr (BIAS) v += bv;
        if (b0 + k2 < B) stg128f_nt(y + (b0 + k2) * N16 + 4 * lane, v);
    }
}

// W[block][row][col] -> transposed operand order: dst[block][lane] = W[block][4 * (lane / 16) + u][lane % 16], u = 0..3
template <int NT>
__device__ __forceinline__ void stage_weights_t(const float* __restrict__ W, unsigned char* dst, int tid)
{
    constexpr int PER = 16 * 64 / NT;
    f32x4 v[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int e = tid + k * NT, blk = e >> 6, lane = e & 63;
        const float* p = W + ((size_t)blk * 16 + 4 * (lane >> 4)) * 16 + (lane & 15);
        v[k] = f32x4{p[0], p[16], p[32], p[48]};
    }
#pragma unroll
    for (int k = 0; k < PER; ++k) *reinterpret_cast<f32x4*>(dst + (size_t)(tid + k * NT) * 16) = v[k];
}

// Transposed multiply y = x M for the same shape: the two dx stages of the backward kernel below on
// their own (x plays the part of dy), in the forward kernel's persistent eight-wave form.
//   dY1[b][kk = r][j = c] = sum_l L[c][l][r] x[b][16l + c]      -> tile [b][j][kk]
//   y[b][16kk + i]        = sum_j R[kk][j][i] dY1[b][kk][j]     -> tile (row-major), full-row stores
__global__ void __launch_bounds__(512)
fwd_t_sq16_kernel(const float* __restrict__ x, const float* __restrict__ R, const float* __restrict__ L,
                  float* __restrict__ y, int64_t B, int64_t ntiles)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ldsb[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int bl = lane & 15, h = lane >> 4;
    unsigned char* RTop = ldsb;
    unsigned char* LTop = ldsb + SQ16_W_BYTES;
    unsigned char* T = ldsb + 2 * SQ16_W_BYTES + (size_t)wave * SQ16_T_BYTES;
    const int64_t stride = (int64_t)gridDim.x * SQ16_WAVES;
    int64_t tile = (int64_t)blockIdx.x * SQ16_WAVES + wave;
    // The operand of the first stage is xa[v] = x[b][64h + 4v .. +3] (element 16u + c is W[b][c][l = 4h + u]):
    // 256 contiguous bytes per lane, which as direct loads would touch 64 cache lines per instruction.
    // The rows are loaded one full 1 KiB row per instruction instead and turned through the tile.
    auto load_rows = [&](int64_t tl, f32x4 (&raw)[16]) {
#pragma unroll
        for (int k2 = 0; k2 < 16; ++k2) {
            int64_t row = tl * 16 + k2;
            row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
            raw[k2] = ldg128f_nt(x + row * N16 + 4 * lane);
        }
    };
    f32x4 raw[16];
    if (tile < ntiles) load_rows(tile, raw);  // in flight while the weights are staged
    stage_weights_t<512>(R, RTop, tid);
    stage_weights_t<512>(L, LTop, tid);
    __syncthreads();
    for (; tile < ntiles; tile += stride) {
#pragma unroll
        for (int k2 = 0; k2 < 16; ++k2) *reinterpret_cast<f32x4*>(T + t_off(k2, lane)) = raw[k2];
        const int64_t next = tile + stride;
        if (next < ntiles) load_rows(next, raw);  // the next tile's rows are fetched early
        wave_lds_fence();
        f32x4 xa[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) xa[v] = *reinterpret_cast<const f32x4*>(T + t_off(bl, 16 * h + v));
        wave_lds_fence();  // every lane has its operand: the tile is reused for dY1
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const f32x4 la = *reinterpret_cast<const f32x4*>(LTop + ((size_t)c * 64 + lane) * 16);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma4(la[u], xa[4 * u + (c >> 2)][c & 3], acc);
            *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * c + h)) = acc;
        }
        wave_lds_fence();
        // lane (b, h): dY1[b][kk][j = 4h + u], four kk per read
        f32x4 db[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) db[u][v] = *reinterpret_cast<const f32x4*>(T + t_off(bl, 4 * (4 * h + u) + v));
        wave_lds_fence();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const f32x4 rt = *reinterpret_cast<const f32x4*>(RTop + ((size_t)kk * 64 + lane) * 16);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma4(rt[u], db[u][kk >> 2][kk & 3], acc);
            *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * kk + h)) = acc;
        }
        wave_lds_fence();
        const int64_t b0 = tile * 16;
#pragma unroll
        for (int k2 = 0; k2 < 16; ++k2) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(T + t_off(k2, lane));
            if (b0 + k2 < B) stg128f_nt(y + (b0 + k2) * N16 + 4 * lane, v);
        }
        wave_lds_fence();
    }
}

// Backward: one persistent kernel for dx, dR and dL (adjoints of steps 3, 2, P^T, 1 of Section 3.3;
// the paper leaves them to automatic differentiation, Section 4).  4 waves per workgroup, one per
// SIMD, so that a wave can keep both weight gradients (2 x 4096 fp32 = 128 registers per lane) in
// MFMA accumulators for the whole launch next to its operands.  Per 16-row tile a wave runs five
// groups of 64 MFMAs; its LDS tile is reused between them for the re-layouts:
//   1. Y1 = step 1 (recomputed)                            -> tile [b][kk][j]
//   2. dL[c][l][r] += sum_b dy[b][16l + c] Y1[b][r][c]      contraction over the 16 rows: operands
//      are read "down the rows" (lane = l resp. r, K-slot = row), 16 bytes = four blocks c at once
//   3. dU[b][c][r] = sum_l L[c][l][r] dy[b][16l + c], i.e. dY1[b][kk = r][j = c] -> tile [b][j][kk]
//   4. dR[kk][j][i] += sum_b dY1[b][kk][j] x[b][16kk + i]   (x re-laid as tile [b][i][kk])
//   5. dx[b][16kk + i] = sum_j R[kk][j][i] dY1[b][kk][j]    -> tile, then full-row stores
// The per-wave gradients go to the workspace and are summed by `reduce_sq16_kernel`.
constexpr int SQ16B_WAVES = 4;
constexpr size_t SQ16B_LDS = 4 * SQ16_W_BYTES + SQ16B_WAVES * SQ16_T_BYTES;  // 128 KiB

__global__ void __launch_bounds__(256)
bwd_sq16_kernel(const float* __restrict__ dy, const float* __restrict__ x, const float* __restrict__ R,
                const float* __restrict__ L, float* __restrict__ dx, float* __restrict__ P, int64_t B, int64_t ntiles)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ldsb[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int bl = lane & 15, h = lane >> 4;
    unsigned char* Rop = ldsb;                         // R[kk][j = lane%16][i = 4h + u]
    unsigned char* RTop = ldsb + SQ16_W_BYTES;         // R[kk][j = 4h + u][i = lane%16]
    unsigned char* LTop = ldsb + 2 * SQ16_W_BYTES;     // L[c][l = 4h + u][r = lane%16]
    unsigned char* T = ldsb + 3 * SQ16_W_BYTES + (size_t)wave * SQ16_T_BYTES;
    f32x4 accR[16], accL[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) {
        accR[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        accL[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const int64_t stride = (int64_t)gridDim.x * SQ16B_WAVES;
    int64_t tile = (int64_t)blockIdx.x * SQ16B_WAVES + wave;
    auto load_x = [&](int64_t tl, f32x4 (&xa)[16]) {
        int64_t row = tl * 16 + bl;
        row = row < B ? row : B - 1;
        const float* p = x + row * N16 + 4 * h;
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) xa[kk] = ldg128f_nt(p + 16 * kk);
    };
    // dya[v] = dy[b][64h + 4v .. +3]: element 16u + c is dW[b][c][l = 4h + u]; rows past the end count as zero
    auto load_dy = [&](int64_t tl, f32x4 (&dya)[16]) {
        int64_t row = tl * 16 + bl;
        const float m = row < B ? 1.f : 0.f;
        row = row < B ? row : B - 1;
        const float* p = dy + row * N16 + 64 * h;
#pragma unroll
        for (int v = 0; v < 16; ++v) dya[v] = *reinterpret_cast<const f32x4*>(p + 4 * v) * m;
    };
    // daq[cq][u] = dy[b0 + 4h + u][16*bl + 4cq .. +3]: the same rows "down the batch" for the dL product (read back from the tile)
    f32x4 xa[16], dya[16], daq[4][4];
    if (tile < ntiles) {  // in flight while the weights are staged
        load_x(tile, xa);
        load_dy(tile, dya);
    }
    stage_weights<256>(R, Rop, tid);
    stage_weights_t<256>(R, RTop, tid);
    stage_weights_t<256>(L, LTop, tid);
    __syncthreads();
    for (; tile < ntiles; tile += stride) {
        const int64_t b0 = tile * 16;
        const int64_t next = tile + stride;
        // the dL product wants the same dy rows "down the batch": turned through the wave's tile (free at
        // this point) instead of a second look at global memory
#pragma unroll
        for (int v = 0; v < 16; ++v) *reinterpret_cast<f32x4*>(T + t_off(bl, 16 * h + v)) = dya[v];
        wave_lds_fence();
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int cq = 0; cq < 4; ++cq) daq[cq][u] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + cq));
        wave_lds_fence();
        // ---- 1. Y1[b][kk][j = 4h + i] -> tile [b][kk][j]
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const f32x4 ra = *reinterpret_cast<const f32x4*>(Rop + ((size_t)kk * 64 + lane) * 16);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma4(ra[u], xa[kk][u], acc);
            *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * kk + h)) = acc;
        }
        wave_lds_fence();
        // ---- 2. dL: A lane (l, h) = dy[b0 + 4h + u][16l + c], B lane (r, h) = Y1[b0 + 4h + u][r][c]
#pragma unroll
        for (int cq = 0; cq < 4; ++cq) {
            f32x4 ub[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) ub[u] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + cq));
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int u = 0; u < 4; ++u) accL[4 * cq + e] = mfma4(daq[cq][u][e], ub[u][e], accL[4 * cq + e]);
        }
        wave_lds_fence();  // Y1 has been read: the tile is reused
        // ---- 3. dY1[b][kk = 4h + i][j = c] -> tile [b][j][kk]
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const f32x4 la = *reinterpret_cast<const f32x4*>(LTop + ((size_t)c * 64 + lane) * 16);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma4(la[u], dya[4 * u + (c >> 2)][c & 3], acc);
            *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * c + h)) = acc;
        }
        if (next < ntiles) load_dy(next, dya);  // the next tile's rows are fetched early
        wave_lds_fence();
        // operands of 4 (lane (j, h): dY1[b0 + 4h + u][kk][j], four kk per read) and of 5
        // (lane (b, h): dY1[b][kk][j = 4h + u], four kk per read)
        f32x4 a2[4][4], db[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                a2[u][v] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + v));
                db[u][v] = *reinterpret_cast<const f32x4*>(T + t_off(bl, 4 * (4 * h + u) + v));
            }
        wave_lds_fence();
        // x re-laid as tile [b][i][kk]
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * (4 * h + e) + v)) =
                    f32x4{xa[4 * v][e], xa[4 * v + 1][e], xa[4 * v + 2][e], xa[4 * v + 3][e]};
        if (next < ntiles) load_x(next, xa);
        wave_lds_fence();
        // ---- 4. dR: B lane (i, h) = x[b0 + 4h + u][16kk + i]
#pragma unroll
        for (int kq = 0; kq < 4; ++kq) {
            f32x4 xb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) xb[u] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + kq));
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int u = 0; u < 4; ++u) accR[4 * kq + e] = mfma4(a2[u][kq][e], xb[u][e], accR[4 * kq + e]);
        }
        wave_lds_fence();
        // ---- 5. dx[b][16kk + 4h + i] -> tile (row-major), then one full row per store instruction
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const f32x4 rt = *reinterpret_cast<const f32x4*>(RTop + ((size_t)kk * 64 + lane) * 16);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = mfma4(rt[u], db[u][kk >> 2][kk & 3], acc);
            *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * kk + h)) = acc;
        }
        wave_lds_fence();
#pragma unroll
        for (int k2 = 0; k2 < 16; ++k2) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(T + t_off(k2, lane));
            if (b0 + k2 < B) stg128f_nt(dx + (b0 + k2) * N16 + 4 * lane, v);
        }
        wave_lds_fence();
    }
    // per-wave gradients: P[wave id][0][kk][j][i], P[wave id][1][c][l][r]; acc[e] is row 4h + e, column lane % 16
    float* Pw = P + ((size_t)blockIdx.x * SQ16B_WAVES + wave) * 8192;
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            Pw[t * 256 + (4 * h + e) * 16 + bl] = accR[t][e];
            Pw[4096 + t * 256 + (4 * h + e) * 16 + bl] = accL[t][e];
        }
}

// Backward with one workgroup per 16-row tile, for batches of up to 1024 tiles: the five MFMA groups of the tile
// are split over four waves (wave q), each taking a quarter of every group's sixteen blocks -- block kk or c in
// 4q .. 4q+3 -- so a tile takes a quarter of the time it takes one wave and the tiles of a short batch run on
// different CUs; the weights come straight from global memory in operand order (no staging pass) and every wave
// holds only its quarter of the operands (4 of the 16 pieces of x and dy) and of the gradients.  The exchanges
// through the tile are the ones of bwd_sq16_kernel, with workgroup barriers in place of the wave fences.  Every
// workgroup writes its tile's gradients to P[tile][8192] and reduce_sq16_kernel sums them in tile order.  Each
// workgroup reads all of R and L (48 KiB against 32 KiB of activations), which is why long batches take the
// persistent kernel.
constexpr int64_t SQ16T_TILES = 1024;

__global__ void __launch_bounds__(256)
bwd_sq16_tile_kernel(const float* __restrict__ dy, const float* __restrict__ x, const float* __restrict__ R,
                      const float* __restrict__ L, float* __restrict__ dx, float* __restrict__ P,
                     int64_t B)
{
    __shared__ __attribute__((aligned(16))) unsigned char T[SQ16_T_BYTES];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int q = wave;
    const int bl = lane & 15, h = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * 16;
    int64_t row = b0 + bl;
    const float msk = row < B ? 1.f : 0.f;  // rows past the end count as zero in dy (and are computed from a valid row of x)
    row = row < B ? row : B - 1;
    // this wave's quarter of the tile's operands: x[b][16kk + 4h ..] for kk = 4q + w; dy[b][64h + 4(4u + q) ..] for u = 0..3
    f32x4 xa[4], dya[4], ra[4], rt[4], lt[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) xa[w] = ldg128f_nt(x + row * N16 + 16 * (4 * q + w) + 4 * h);
#pragma unroll
    for (int u = 0; u < 4; ++u) dya[u] = *reinterpret_cast<const f32x4*>(dy + row * N16 + 64 * h + 4 * (4 * u + q)) * msk;
    // weights in operand order, blocks 4q .. 4q+3: R[kk][j = bl][i = 4h + u];  R[kk][j = 4h + u][i = bl];  L[c][l = 4h + u][r = bl]
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int blk = 4 * q + w;
        ra[w] = *reinterpret_cast<const f32x4*>(R + ((size_t)blk * 16 + bl) * 16 + 4 * h);
        const float* pr = R + ((size_t)blk * 16 + 4 * h) * 16 + bl;
        rt[w] = f32x4{pr[0], pr[16], pr[32], pr[48]};
        const float* pl = L + ((size_t)blk * 16 + 4 * h) * 16 + bl;
        lt[w] = f32x4{pl[0], pl[16], pl[32], pl[48]};
    }
    __builtin_amdgcn_sched_barrier(0);  // every load is issued before the first use
    // dy "down the batch" for the dL product: through the tile
#pragma unroll
    for (int u = 0; u < 4; ++u) *reinterpret_cast<f32x4*>(T + t_off(bl, 16 * h + 4 * u + q)) = dya[u];
    __syncthreads();
    f32x4 daq[4];  // daq[u] = dy[b0 + 4h + u][16 bl + 4q .. +3]
#pragma unroll
    for (int u = 0; u < 4; ++u) daq[u] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + q));
    __syncthreads();
    // ---- 1. Y1[b][kk][j = 4h + i] -> tile [b][kk][j], kk = 4q + w
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = mfma4(ra[w][u], xa[w][u], acc);
        *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * (4 * q + w) + h)) = acc;
    }
    __syncthreads();
    // ---- 2. dL[c = 4q + e][l][r] += sum_b dy[b][16l + c] Y1[b][r][c]
    f32x4 accL[4], accR[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) accL[e] = accR[e] = f32x4{0.f, 0.f, 0.f, 0.f};
    {
        f32x4 ub[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) ub[u] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + q));
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int u = 0; u < 4; ++u) accL[e] = mfma4(daq[u][e], ub[u][e], accL[e]);
    }
    __syncthreads();  // Y1 has been read: the tile is reused
    // ---- 3. dY1[b][kk = 4h + i][j = c] -> tile [b][j][kk], c = 4q + w (dW[b][c][l = 4h + u] = dya[u][w])
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = mfma4(lt[w][u], dya[u][w], acc);
        *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * (4 * q + w) + h)) = acc;
    }
    __syncthreads();
    // operands of 4 (lane (j, h): dY1[b0 + 4h + u][kk = 4q + e][j]) and of 5 (lane (b, h): dY1[b][kk = 4q + e][j = 4h + u])
    f32x4 a2[4], db[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        a2[u] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + q));
        db[u] = *reinterpret_cast<const f32x4*>(T + t_off(bl, 4 * (4 * h + u) + q));
    }
    __syncthreads();
    // x re-laid as tile [b][i][kk]: this wave holds kk = 4q .. 4q+3, i = 4h + e
#pragma unroll
    for (int e = 0; e < 4; ++e)
        *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * (4 * h + e) + q)) = f32x4{xa[0][e], xa[1][e], xa[2][e], xa[3][e]};
    __syncthreads();
    // ---- 4. dR[kk = 4q + e][j][i] += sum_b dY1[b][kk][j] x[b][16kk + i]
    {
        f32x4 xb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) xb[u] = *reinterpret_cast<const f32x4*>(T + t_off(4 * h + u, 4 * bl + q));
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int u = 0; u < 4; ++u) accR[e] = mfma4(a2[u][e], xb[u][e], accR[e]);
    }
    __syncthreads();
    // ---- 5. dx[b][16kk + 4h + i], kk = 4q + w -> tile (row-major), then one full row per store instruction
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = mfma4(rt[w][u], db[u][w], acc);
        *reinterpret_cast<f32x4*>(T + t_off(bl, 4 * (4 * q + w) + h)) = acc;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int k2 = 4 * q + w;
        const f32x4 v = *reinterpret_cast<const f32x4*>(T + t_off(k2, lane));
        if (b0 + k2 < B) stg128f_nt(dx + (b0 + k2) * N16 + 4 * lane, v);
    }
    // this wave's quarter of the tile's gradients: P[tile][dR then dL][block][row][column]
    float* Pt = P + (size_t)blockIdx.x * 8192;
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // accR[e] is block kk = 4q + e, accL[e] block c = 4q + e; element i is row 4h + i, column bl
            Pt[(4 * q + e) * 256 + (4 * h + i) * 16 + bl] = accR[e][i];
            Pt[4096 + (4 * q + e) * 256 + (4 * h + i) * 16 + bl] = accL[e][i];
        }
}

// out[e] = sum_z P[z][e] for the 8192 gradient entries (dR then dL); 16 entries x 16 z-lanes per block
__global__ void __launch_bounds__(256)
reduce_sq16_kernel(const float* __restrict__ P, float* __restrict__ dR, float* __restrict__ dL, int nz)
{
    __shared__ float part[16][17];
    const int el = threadIdx.x & 15, zl = threadIdx.x >> 4;
    const int e = blockIdx.x * 16 + el;
    float s = 0.f;
    int z = zl;
    for (; z + 16 * 7 < nz; z += 16 * 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = P[(size_t)(z + 16 * u) * 8192 + e];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; z < nz; z += 16) s += P[(size_t)z * 8192 + e];
    part[zl][el] = s;
    __syncthreads();
    if (zl == 0) {
        float tot = 0.f;
#pragma unroll
        for (int k = 0; k < 16; ++k) tot += part[k][el];
        if (e < 4096) dR[e] = tot;
        else dL[e - 4096] = tot;
    }
}

int bwd_sq16_grid(const Problem& pb)
{
    const int64_t ntiles = (pb.B + 15) / 16;
    int64_t grid = (ntiles + SQ16B_WAVES - 1) / SQ16B_WAVES;
    if (grid > 256) grid = 256;  // one persistent workgroup per CU
    if (grid < 1) grid = 1;
    return (int)grid;
}

}  // namespace

constexpr int64_t kSmallTiles = 2048;  // forward: batches of at most this many 16-row tiles take the one-workgroup-per-tile kernel

bool sq16_supported(const Problem& pb)
{
    // both readings of the mid permutation coincide when k = q
    return pb.dtype == 0 && pb.k == 16 && pb.p == 16 && pb.q == 16 && pb.s == 16;
}

int fwd_t_sq16(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if (!sq16_supported(pb)) return -2;
    auto kern = fwd_t_sq16_kernel;
    if (allow_dynamic_lds((const void*)kern, SQ16_LDS) != hipSuccess)
        return -4;
    const int64_t ntiles = (pb.B + 15) / 16;
    int64_t grid = (ntiles + SQ16_WAVES - 1) / SQ16_WAVES;
    if (grid > 256) grid = 256;  // one persistent workgroup per CU
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ16_LDS, st, (const float*)x, (const float*)R,
                       (const float*)L, (float*)y, pb.B, ntiles);
    return hip_status(hipGetLastError());
}

int fwd_sq16(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if (!sq16_supported(pb)) return -2;
    const int64_t ntiles = (pb.B + 15) / 16;
    if (ntiles <= kSmallTiles) {  // one four-wave workgroup per tile, no weight staging
        auto tk = pb.bias ? fwd_sq16_tile_kernel<true> : fwd_sq16_tile_kernel<false>;
        hipLaunchKernelGGL(tk, dim3((unsigned)ntiles), dim3(256), 0, st, (const float*)x, (const float*)R,
                           (const float*)L, (const float*)pb.bias, (float*)y, pb.B);
        return hip_status(hipGetLastError());
    }
    auto kern = pb.bias ? fwd_sq16_kernel<true> : fwd_sq16_kernel<false>;
    if (allow_dynamic_lds((const void*)kern, SQ16_LDS) != hipSuccess)
        return -4;
    int64_t grid = (ntiles + SQ16_WAVES - 1) / SQ16_WAVES;
    if (grid > 256) grid = 256;  // one persistent workgroup per CU
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ16_LDS, st, (const float*)x, (const float*)R,
                       (const float*)L, (const float*)pb.bias, (float*)y, pb.B, ntiles);
    return hip_status(hipGetLastError());
}

}  // namespace monarch

namespace monarch {

size_t bwd_sq16_workspace(const Problem& pb) { return (size_t)bwd_sq16_grid(pb) * SQ16B_WAVES * 8192 * sizeof(float); }

int bwd_sq16(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx,
             void* dR, void* dL, void* ws, hipStream_t st)
{
    if (!sq16_supported(pb)) return -2;
    if (pb.B == 0) {
        const int rc = launch_fill_zero_f32((float*)dR, pb.n_R(), st);
        return rc ? rc : launch_fill_zero_f32((float*)dL, pb.n_L(), st);
    }
    const int grid = bwd_sq16_grid(pb);
    const int64_t ntiles = (pb.B + 15) / 16;
    if (ntiles <= SQ16T_TILES) {  // one workgroup per tile, then the sum over tiles
        if ((size_t)ntiles * 8192 * sizeof(float) > bwd_sq16_workspace(pb)) return -2;
        hipLaunchKernelGGL(bwd_sq16_tile_kernel, dim3((unsigned)ntiles), dim3(256), 0, st, (const float*)dy, (const float*)x,
                           (const float*)R, (const float*)L, (float*)dx, (float*)ws, pb.B);
        if (hipGetLastError() != hipSuccess) return -4;
        hipLaunchKernelGGL(reduce_sq16_kernel, dim3(8192 / 16), dim3(256), 0, st, (const float*)ws, (float*)dR, (float*)dL,
                           (int)ntiles);
        return hip_status(hipGetLastError());
    }
    auto kern = bwd_sq16_kernel;
    if (allow_dynamic_lds((const void*)kern, SQ16B_LDS) != hipSuccess)
        return -4;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), SQ16B_LDS, st, (const float*)dy, (const float*)x, (const float*)R,
                       (const float*)L, (float*)dx, (float*)ws, pb.B, ntiles);
    if (hipGetLastError() != hipSuccess) return -4;
    hipLaunchKernelGGL(reduce_sq16_kernel, dim3(8192 / 16), dim3(256), 0, st, (const float*)ws, (float*)dR, (float*)dL,
                       grid * SQ16B_WAVES);
    return hip_status(hipGetLastError());
}

}  // namespace monarch
