// bf16 kernels for the square Monarch matrix of Definition 3.1 with m = 64 (n = 4096,
// k = q = s = p = 64): fused forward, and the backward data path.
//
// Per batch row the input is a 64 x 64 matrix X[kk][i].  Step 1 of Section 3.3 multiplies
// row kk by R[kk], the permutation turns the result Y1[kk][j] into U[c][r] = Y1[r][c], step 2
// multiplies row c of U (column c of Y1) by L[c], and step 3 writes y[l*64 + c] = W[c][l].  So
// every output block needs one column from every input block: a workgroup has to own whole rows,
// 8 KiB each in bf16.  A workgroup (8 waves) owns 32 rows.
//
// "Block stage": wave w multiplies blocks 8w .. 8w+7 of a block-diagonal factor with its rows and
// keeps the 32 x 512 results packed in registers (pairs of blocks per dword), because the full
// 256 KiB intermediate does not fit in LDS.  The intermediate is exchanged in two halves (output
// columns < 32, then >= 32): a half is written to LDS as T[b][col][block] (block fastest, 16-byte
// writes of the wave's eight blocks), which is exactly the operand order of the next factor for
// its block number `col`: the transposition P^T costs no data movement of its own.
//
// "Column stage": wave (cg, lt) multiplies the eight blocks 32h + 8cg .. +7 of the next factor,
// output rows 32lt .. 32lt+31, with the half in LDS.
//
// MFMA operands are loaded from global memory in operand layout.  Which contraction index sits
// in which K-slot is free as long as both operands agree, so lane group g of K-step u takes
// indices 32g + 8u .. +7: every lane then reads 64 contiguous bytes of its row.
// Everything that goes back to global memory is first transposed through LDS so that it is
// written in full 128-byte lines (16-byte pieces scattered over lines cost 2-3x the time).
//
// Backward (adjoints of steps 3, 2, P^T, 1; the paper leaves them to automatic differentiation,
// Section 4):
//   transpose   dW[b][c][l] = dy[b][l*64 + c]  (adjoint of step 3, a pure permutation) and the
//               transposed weights LT[c][r][l], RT[kk][i][j]: batched 64 x 64 transposes.
//   data        block stage (x, R) -> U to the workspace (dL needs it);
//               block stage (dW, LT) -> dU[b][c][r] = dY1[b][r][c], exchanged like the forward
//               intermediate and also copied to the workspace (dR needs it);
//               column stage (RT) -> dx.
//   wgrad       dL = sum_b dW (x) U and dR = sum_b dY1 (x) x as batch-contracted GEMMs with 64
//               groups (monarch_mfma_wgrad.hip).
#include "monarch_internal.h"
#include "monarch_mfma_common.h"

namespace monarch {

namespace {

constexpr int M64 = 64, N64 = 4096;
constexpr int SQ_BM = 32;                          // rows per workgroup
constexpr int SQ_ROWB = 32 * 128 + 16;             // bytes per row of the exchange buffer (32 cols x 64 blocks + pad)
constexpr size_t SQ_LDS = (size_t)SQ_BM * SQ_ROWB; // 131584 bytes

struct Lane {
    int wave, lane, ln, g;
};

// Block stage.  act: the lane's row, at column 32*g; W[block][out][in] (64 x 64 each).
// Results: bf16 pairs (block even, block odd) of T[b = ln][block][col], col = 32*jt + 8*(i/4) + 4*g + i%4.
// The half col < 32 goes to the exchange buffer as it is produced (LDS must be idle), the half
// col >= 32 is returned in pk1[i][t2].
// PACKED: W is the factor in fragment order (pack64_kernel): a weight operand is then one contiguous
// 1 KiB read per wave instruction instead of 32 lines touched twice.
template <bool PACKED>
__device__ __forceinline__ void block_stage(const Lane& t_, const uint16_t* __restrict__ act_row,
                                            const uint16_t* __restrict__ W, unsigned char* ldsb, u32x4 (&pk1)[16])
{
    const int wave = t_.wave, ln = t_.ln, g = t_.g;
    const uint16_t* arow = act_row + (size_t)wave * 8 * M64;
    const uint16_t* Wrow = PACKED ? W + ((size_t)wave * 8 * 8 * 64 + t_.lane) * 8
                                  : W + ((size_t)wave * 8 * M64 + ln) * M64 + 32 * g;
    u32x4 xa[2][4], ra[2][4];
    auto load_x = [&](int t, int s) {
#pragma unroll
        for (int u = 0; u < 4; ++u) xa[s][u] = ldg128(arow + t * M64 + 8 * u);
    };
    auto load_r = [&](int t, int jt) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            ra[jt][u] = PACKED ? ldg128(Wrow + (size_t)((t * 2 + jt) * 4 + u) * 512)
                               : ldg128(Wrow + ((size_t)t * M64 + 32 * jt) * M64 + 8 * u);
    };
    load_x(0, 0);
    load_r(0, 0);
    load_r(0, 1);
    f32x16 ev[2];
    u32x2 q0[16];
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
                for (int i = 0; i < 16; ++i) pk1[i][t >> 1] = pack_bf16x2(ev[1][i], acc[i]);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) q0[i][(t >> 1) & 1] = pack_bf16x2(ev[0][i], acc[i]);
                if ((t & 3) == 3) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int jl = 8 * (i >> 2) + 4 * g + (i & 3);
                        *reinterpret_cast<u32x2*>(ldsb + (size_t)ln * SQ_ROWB + jl * 128 + 16 * wave + 8 * (t >> 2)) =
                            q0[i];
                    }
                }
            }
        }
    }
}

// second half of the block-stage results -> exchange buffer
__device__ __forceinline__ void exchange_write(const Lane& t_, unsigned char* ldsb, const u32x4 (&pk1)[16])
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int jl = 8 * (i >> 2) + 4 * t_.g + (i & 3);
        *reinterpret_cast<u32x4*>(ldsb + (size_t)t_.ln * SQ_ROWB + jl * 128 + 16 * t_.wave) =
            pk1[i];
    }
}

// Column stage for half h: eight blocks c = 32h + 8cg + cc of W2[c][out][in], output tile lt.
// acc(cc) = D[out = 32*lt + 8*(i/4) + 4*g + i%4][b = ln]; `sink(cc, acc)` consumes it.
template <bool PACKED, typename Sink>
__device__ __forceinline__ void column_stage(const Lane& t_, const uint16_t* __restrict__ W2, const unsigned char* ldsb,
                                             int h, Sink&& sink)
{
    const int cg = t_.wave & 3, lt = t_.wave >> 2;
    const unsigned char* ub = ldsb + (size_t)t_.ln * SQ_ROWB + (8 * cg) * 128 + 64 * t_.g;
    // packed: fragment (block c, tile lt, K-step u) at ((c*2 + lt)*4 + u) * 512 elements, + lane * 8
    const uint16_t* Wrow = PACKED ? W2 + ((size_t)((32 * h + 8 * cg) * 2 + lt) * 4 * 64 + t_.lane) * 8
                                  : W2 + (((size_t)(32 * h + 8 * cg)) * M64 + 32 * lt + t_.ln) * M64 + 32 * t_.g;
    constexpr size_t BLK = PACKED ? 8 * 512 : (size_t)M64 * M64;  // elements between consecutive blocks c
    constexpr size_t KST = PACKED ? 512 : 8;                       // elements between consecutive K-steps u
    u32x4 la[2][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) la[0][u] = ldg128(Wrow + u * KST);
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) {
        const int s = cc & 1;
        __builtin_amdgcn_sched_barrier(0);
        if (cc + 1 < 8) {
#pragma unroll
            for (int u = 0; u < 4; ++u) la[s ^ 1][u] = ldg128(Wrow + (size_t)(cc + 1) * BLK + u * KST);
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
        sink(cc, acc);
    }
}

// Column stage of the backward for half h, in place: wave w multiplies the four blocks c = 32h + 4w + cc of the packed
// factor W2 (both 32-row output tiles) with line (b, 4w + cc) of the exchange buffer and writes the 64 results over that
// same line: out[b][4w + cc][i], 128 bytes.  Every lane reads and writes its own row b = ln only and no other wave
// touches these four lines, so the order of one wave's LDS operations is all the synchronisation the overwrite needs;
// the results never wait in registers for the buffer to die (64 registers, which the kernel otherwise spills).
__device__ __forceinline__ void column_stage_inplace(const Lane& t_, const uint16_t* __restrict__ W2, unsigned char* ldsb, int h)
{
    unsigned char* line0 = ldsb + (size_t)t_.ln * SQ_ROWB + (4 * t_.wave) * 128;
    // fragment (block c, tile lt, K-step u) at ((c*2 + lt)*4 + u) * 512 elements, + lane * 8: the eight (block, tile)
    // steps of this wave are contiguous, n = 2*cc + lt
    const uint16_t* Wrow = W2 + ((size_t)(32 * h + 4 * t_.wave) * 2 * 4 * 64 + t_.lane) * 8;
    u32x4 la[2][4], ua[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) la[0][u] = ldg128(Wrow + (size_t)u * 512);
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        const int cc = n >> 1, lt = n & 1, s = n & 1;
        unsigned char* line = line0 + cc * 128;
        __builtin_amdgcn_sched_barrier(0);
        if (n + 1 < 8) {
#pragma unroll
            for (int u = 0; u < 4; ++u) la[s ^ 1][u] = ldg128(Wrow + (size_t)((n + 1) * 4 + u) * 512);
        }
        if (lt == 0) {  // the operand line is read once, before either tile's results are written over it
#pragma unroll
            for (int u = 0; u < 4; ++u) ua[u] = *reinterpret_cast<const u32x4*>(line + 64 * t_.g + 16 * u);
        }
        __builtin_amdgcn_sched_barrier(0);
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = mfma32(as_bf16x8(la[s][u]), as_bf16x8(ua[u]), acc);
        // acc[i] = D[out = 32*lt + 8*(i/4) + 4*g + i%4][b = ln]
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
            *reinterpret_cast<u32x2*>(line + (32 * lt + 8 * i4 + 4 * t_.g) * 2) =
                u32x2{pack_bf16x2(acc[4 * i4], acc[4 * i4 + 1]), pack_bf16x2(acc[4 * i4 + 2], acc[4 * i4 + 3])};
    }
}

// Copies a 32 x 32-line LDS tile to global memory in full lines: wave w takes rows b = 4w..4w+3,
// 128 lines, eight per instruction (1 KiB contiguous).  Line (b, jl) goes to
// dst[(b0 + b) * 4096 + (col0 + jl) * 64 ..].  SWZ: tile rows are 4096 bytes and the 16-byte piece
// index is XOR-ed with b % 8; otherwise rows are SQ_ROWB bytes, pieces in order.
template <bool SWZ, bool NT = SWZ>
__device__ __forceinline__ void copy_out(const Lane& t_, const unsigned char* ldsb, uint16_t* __restrict__ dst,
                                         int64_t b0, int64_t B, int col0)
{
#pragma unroll
    for (int k2 = 0; k2 < 16; ++k2) {
        const int line = 8 * k2 + (t_.lane >> 3), pc = t_.lane & 7;
        const int b = 4 * t_.wave + (line >> 5), jl = line & 31;
        const unsigned char* src = SWZ ? ldsb + (size_t)b * 4096 + jl * 128 + ((pc ^ (b & 7)) * 16)
                                       : ldsb + (size_t)b * SQ_ROWB + jl * 128 + pc * 16;
        const u32x4 v = *reinterpret_cast<const u32x4*>(src);
        if (b0 + b < B) {
            uint16_t* p = dst + (b0 + b) * N64 + (size_t)(col0 + jl) * M64 + 8 * pc;
            if (NT) stg128_nt(p, v);  // final outputs: streamed; workspace copies stay cacheable for the next kernel
            else *reinterpret_cast<u32x4*>(p) = v;
        }
    }
}

__device__ __forceinline__ Lane make_lane()
{
    const int tid = threadIdx.x;
    Lane t;
    t.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    t.lane = tid & 63;
    t.ln = t.lane & 31;
    t.g = t.lane >> 5;
    return t;
}

// ------------------------------------------------------------------------ forward ----

template <bool PACKED>
__global__ void __launch_bounds__(512)
fwd_sq64_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ R,
                const uint16_t* __restrict__ L, uint16_t* __restrict__ y, int64_t B)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ldsb[];
    const Lane t = make_lane();
    const int ln = t.ln, g = t.g;
    const int64_t b0 = (int64_t)blockIdx.x * SQ_BM;
    int64_t row = b0 + ln;
    row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped

    // step 1: Y1[b][kk][j] -> exchange layout T[b][j][kk]
    u32x4 pk1[16];  // pk1[i][t]: one 16-byte exchange piece per i, filled component by component
    block_stage<PACKED>(t, x + row * N64 + 32 * g, R, ldsb, pk1);

    // step 2 for the 32 blocks c = j of each half.
    // po[h][c2][i]: bf16 pair (c0 + 2*c2, c0 + 2*c2 + 1) of W[b = ln][c][l], c0 = 32h + 8cg,
    // l = 32*lt + 8*(i/4) + 4*g + i%4
    const int cg = t.wave & 3, lt = t.wave >> 2;
    uint32_t po[2][4][16];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (h) {
            __syncthreads();  // step 2 of the first half has read everything it needs
            exchange_write(t, ldsb, pk1);
        }
        __syncthreads();
        f32x16 ev;
        column_stage<PACKED>(t, L, ldsb, h, [&](int cc, const f32x16& acc) {
            if ((cc & 1) == 0) {
                ev = acc;
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) po[h][cc >> 1][i] = pack_bf16x2(ev[i], acc[i]);
            }
        });
    }

    // step 3: y[b][l*64 + c], transposed through LDS one 32-row tile of l per round.
    // LDS tile: [b][l][8 pieces of 16 B], piece index XOR-ed with b % 8 so that the writes of 8
    // adjacent lanes hit 8 different slots.
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
        copy_out<true>(t, ldsb, y, b0, B, 32 * rnd);
    }
}

// ------------------------------------------------------------------------ pack ----

// A 64-block factor W[blk][out][in] (64 x 64 each) in MFMA fragment order, for up to three factors in
// one launch:  dst[blk][t2][u][lane][e] = W'[blk][32*t2 + lane%32][32*(lane/32) + 8*u + e], where W' = W,
// or W' = W^T per block (tr: the backward multiplies by the transposed factors).  One thread = one
// 16-byte piece; 32768 pieces per factor.
struct Pack64Job { const uint16_t* src; uint16_t* dst; int tr; };
__global__ void __launch_bounds__(256)
pack64_kernel(Pack64Job j0, Pack64Job j1, Pack64Job j2)
{
    const int which = blockIdx.x >> 7;  // 128 blocks of 256 pieces per factor
    const Pack64Job& j = which == 0 ? j0 : (which == 1 ? j1 : j2);
    const int pc = (blockIdx.x & 127) * 256 + threadIdx.x;
    const int lane = pc & 63, ln = lane & 31, g = lane >> 5;
    const int rest = pc >> 6, u = rest & 3, t2 = (rest >> 2) & 1, blk = rest >> 3;
    u32x4 o;
    if (!j.tr) {
        o = ldg128(j.src + ((size_t)blk * M64 + 32 * t2 + ln) * M64 + 32 * g + 8 * u);
    } else {
        const uint16_t* p = j.src + ((size_t)blk * M64 + 32 * g + 8 * u) * M64 + 32 * t2 + ln;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = p[(size_t)e * M64];
#pragma unroll
        for (int w = 0; w < 4; ++w) o[w] = (uint32_t)v[2 * w] | ((uint32_t)v[2 * w + 1] << 16);
    }
    *reinterpret_cast<u32x4*>(j.dst + (size_t)pc * 8) = o;
}

// ------------------------------------------------------------------------ backward ----

// dst[blk][c][r] = src[blk][r][c] for 64 x 64 bf16 blocks; one workgroup (256 threads) per block.
__global__ void __launch_bounds__(256)
transpose64_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst)
{
    __shared__ __attribute__((aligned(16))) uint16_t tile[64][72];  // row stride 144 B
    const int tid = threadIdx.x;
    const uint16_t* s = src + (size_t)blockIdx.x * 4096;
    uint16_t* d = dst + (size_t)blockIdx.x * 4096;
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int e = tid + 256 * it;  // 16-byte piece: row e / 8, columns 8 * (e % 8) ..
        *reinterpret_cast<u32x4*>(&tile[e >> 3][8 * (e & 7)]) = ldg128(s + (size_t)e * 8);
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 2; ++it) {
        const int e = tid + 256 * it;  // output piece: row c = e / 8, columns r0 = 8 * (e % 8) ..
        const int c = e >> 3, r0 = 8 * (e & 7);
        uint32_t v[4];
#pragma unroll
        for (int w = 0; w < 4; ++w)
            v[w] = (uint32_t)tile[r0 + 2 * w][c] | ((uint32_t)tile[r0 + 2 * w + 1][c] << 16);
        *reinterpret_cast<u32x4*>(d + (size_t)e * 8) = u32x4{v[0], v[1], v[2], v[3]};
    }
}

// DX_ONLY: the transposed multiply y = x M on its own (dW is then the transposed input of that
// product): no recompute of step 1, no workspace copies of the intermediates.
template <bool DX_ONLY>
__global__ void __launch_bounds__(512)
bwd_sq64_data_kernel(const uint16_t* __restrict__ dW, const uint16_t* __restrict__ x,
                     const uint16_t* __restrict__ R /* packed */, const uint16_t* __restrict__ LT /* packed L^T */,
                     const uint16_t* __restrict__ RT /* packed R^T */, uint16_t* __restrict__ dx,
                     uint16_t* __restrict__ Uws, uint16_t* __restrict__ dY1ws, int64_t B)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char ldsb[];
    const Lane t = make_lane();
    const int ln = t.ln, g = t.g;
    const int64_t b0 = (int64_t)blockIdx.x * SQ_BM;
    int64_t row = b0 + ln;
    row = row < B ? row : B - 1;

    u32x4 pk1[16];  // pk1[i][t]: one 16-byte exchange piece per i, filled component by component
    // ---- recompute step 1; the exchange layout T[b][j][kk] is U[b][c = j][r = kk]: to the workspace
    if constexpr (!DX_ONLY) {
        block_stage<true>(t, x + row * N64 + 32 * g, R, ldsb, pk1);
        __syncthreads();
        copy_out<false>(t, ldsb, Uws, b0, B, 0);
        __syncthreads();
        exchange_write(t, ldsb, pk1);
        __syncthreads();
        copy_out<false>(t, ldsb, Uws, b0, B, 32);
        __syncthreads();
    }

    // ---- adjoint of step 2: dU[b][c][r] = sum_l LT[c][r][l] dW[b][c][l]; as dY1[b][kk = r][j = c]
    // the exchange layout T[b][r][c] is dY1[b][kk][j]: operand order of the next stage, and the
    // layout of the workspace copy
    block_stage<true>(t, dW + row * N64 + 32 * g, LT, ldsb, pk1);

    // ---- adjoint of step 1: dx[b][kk*64 + i] = sum_j RT[kk][i][j] dY1[b][kk][j], written over the dY1 lines (see
    // column_stage_inplace): line (b, kk) of the buffer becomes dx[b][kk*64 ..], which is also the layout of dx itself
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (h) exchange_write(t, ldsb, pk1);
        __syncthreads();
        if constexpr (!DX_ONLY) {
            copy_out<false>(t, ldsb, dY1ws, b0, B, 32 * h);
            __syncthreads();  // every wave has copied its share of the dY1 half before lines are overwritten
        }
        column_stage_inplace(t, RT, ldsb, h);
        __syncthreads();
        copy_out<false, true>(t, ldsb, dx, b0, B, 32 * h);
        __syncthreads();  // the lines are read before the second half overwrites them
    }
}

// batch chunks of the two weight-gradient GEMMs (64 groups each): about one workgroup per CU
struct Plan64 {
    size_t off_u, off_dy1, off_dw, off_lt, off_rt, off_rp, off_partL, off_partR, total;
    int nz, rows_per_chunk;
    bool ok;
};

void fill_descs64(const Problem& pb, WgradDesc& dl, WgradDesc& dr)
{
    // dL[c][l][r] = sum_b dW[b][c][l] * U[b][c][r];   dR[kk][j][i] = sum_b dY1[b][kk][j] * x[b][kk][i]
    dl = WgradDesc{};
    dl.lda = N64; dl.a_g = M64; dl.deint = 0;
    dl.ldb = N64; dl.b_g = M64; dl.b_seg = 0; dl.seg_w = M64;
    dl.M = M64; dl.N = M64; dl.G = M64; dl.rows = pb.B;
    dr = dl;
}

Plan64 make_plan64(const Problem& pb)
{
    Plan64 pl{};
    WgradDesc dl, dr;
    fill_descs64(pb, dl, dr);
    const int tiles = wgrad_tiles(dl) + wgrad_tiles(dr);
    pl.ok = wgrad_tiles(dl) > 0 && wgrad_tiles(dr) > 0;
    if (!pl.ok) return pl;
    int64_t z = 256 / tiles;  // at most one workgroup per CU: its two LDS buffers leave room for one only
    const int64_t maxz = (pb.B + 255) / 256;
    if (z > maxz) z = maxz;
    if (z < 1) z = 1;
    const int64_t rpc = ((pb.B + z - 1) / z + 63) / 64 * 64;  // whole pipeline rounds (two 32-row steps)
    pl.rows_per_chunk = (int)(rpc > 0 ? rpc : 32);
    pl.nz = (int)((pb.B + pl.rows_per_chunk - 1) / pl.rows_per_chunk);
    if (pl.nz < 1) pl.nz = 1;
    size_t off = 0;
    const size_t act = align_up((size_t)(pb.B > 0 ? pb.B : 1) * N64 * 2, 256);
    pl.off_u = off;   off += act;
    pl.off_dy1 = off; off += act;
    pl.off_dw = off;  off += act;
    pl.off_lt = off;  off += align_up(pb.n_L() * 2, 256);
    pl.off_rt = off;  off += align_up(pb.n_R() * 2, 256);
    pl.off_rp = off;  off += align_up(pb.n_R() * 2, 256);
    pl.off_partL = off; off += align_up((size_t)pl.nz * pb.n_L() * 4, 256);
    pl.off_partR = off; off += align_up((size_t)pl.nz * pb.n_R() * 4, 256);
    pl.total = off;
    return pl;
}

}  // namespace

bool sq64_supported(const Problem& pb)
{
    // both readings of the mid permutation coincide when k = q
    return pb.dtype == 1 && pb.k == 64 && pb.p == 64 && pb.q == 64 && pb.s == 64;
}

int fwd_sq64(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if (!sq64_supported(pb)) return -2;
    auto kern = fwd_sq64_kernel<false>;
    if (allow_dynamic_lds((const void*)kern, SQ_LDS) != hipSuccess)
        return -4;
    const int64_t grid = (pb.B + SQ_BM - 1) / SQ_BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ_LDS, st, (const uint16_t*)x, (const uint16_t*)R,
                       (const uint16_t*)L, (uint16_t*)y, pb.B);
    return hip_status(hipGetLastError());
}

// forward on packed factors: workspace = packed R, then packed L
size_t fwd_sq64_workspace(const Problem& pb) { return align_up(pb.n_R() * 2, 256) + align_up(pb.n_L() * 2, 256); }

int fwd_sq64_ws(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    if (!sq64_supported(pb)) return -2;
    uint16_t* Rp = (uint16_t*)ws;
    uint16_t* Lp = (uint16_t*)((char*)ws + align_up(pb.n_R() * 2, 256));
    if (!pb.ws_packed()) {
        const Pack64Job jr{(const uint16_t*)R, Rp, 0}, jl{(const uint16_t*)L, Lp, 0};
        hipLaunchKernelGGL(pack64_kernel, dim3(2 * 128), dim3(256), 0, st, jr, jl, jl);
        if (hipGetLastError() != hipSuccess) return -4;
    }
    auto kern = fwd_sq64_kernel<true>;
    if (allow_dynamic_lds((const void*)kern, SQ_LDS) != hipSuccess)
        return -4;
    const int64_t grid = (pb.B + SQ_BM - 1) / SQ_BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ_LDS, st, (const uint16_t*)x, Rp, Lp, (uint16_t*)y, pb.B);
    return hip_status(hipGetLastError());
}

bool bwd_sq64_supported(const Problem& pb) { return sq64_supported(pb) && make_plan64(pb).ok; }

// Transposed multiply: input rows re-laid [c][l] (one pass), L^T and R^T packed, then the dx stages.
size_t fwd_t_sq64_workspace(const Problem& pb)
{
    return align_up((size_t)(pb.B > 0 ? pb.B : 1) * N64 * 2, 256) + 2 * align_up((size_t)M64 * M64 * M64 * 2, 256);
}

int fwd_t_sq64(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    if (!sq64_supported(pb)) return -2;
    const int64_t grid = (pb.B + SQ_BM - 1) / SQ_BM;
    if (grid > 0x7fffffffLL || pb.B > 0x7fffffffLL) return -2;
    char* w = (char*)ws;
    uint16_t* xT = (uint16_t*)w;
    uint16_t* LT = (uint16_t*)(w + align_up((size_t)pb.B * N64 * 2, 256));
    uint16_t* RT = LT + align_up((size_t)M64 * M64 * M64 * 2, 256) / 2;
    const Pack64Job jlt{(const uint16_t*)L, LT, 1}, jrt{(const uint16_t*)R, RT, 1};
    hipLaunchKernelGGL(pack64_kernel, dim3(2 * 128), dim3(256), 0, st, jlt, jrt, jrt);
    hipLaunchKernelGGL(transpose64_kernel, dim3((unsigned)pb.B), dim3(256), 0, st, (const uint16_t*)x, xT);
    if (hipGetLastError() != hipSuccess) return -4;
    auto kern = bwd_sq64_data_kernel<true>;
    if (allow_dynamic_lds((const void*)kern, SQ_LDS) != hipSuccess)
        return -4;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ_LDS, st, xT, (const uint16_t*)nullptr,
                       (const uint16_t*)nullptr, LT, RT, (uint16_t*)y, (uint16_t*)nullptr, (uint16_t*)nullptr, pb.B);
    return hip_status(hipGetLastError());
}

size_t bwd_sq64_workspace(const Problem& pb) { return make_plan64(pb).total; }

int bwd_sq64(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx,
             void* dR, void* dL, void* ws, hipStream_t st)
{
    if (!sq64_supported(pb)) return -2;
    const Plan64 pl = make_plan64(pb);
    if (!pl.ok) return -2;
    const bool f32out = pb.wgrad_f32();
    if (pb.B == 0) {
        int rc = f32out ? launch_fill_zero_f32((float*)dR, pb.n_R(), st) : launch_fill_zero_u16((uint16_t*)dR, pb.n_R(), st);
        if (rc) return rc;
        return f32out ? launch_fill_zero_f32((float*)dL, pb.n_L(), st) : launch_fill_zero_u16((uint16_t*)dL, pb.n_L(), st);
    }
    const int64_t grid = (pb.B + SQ_BM - 1) / SQ_BM;
    if (grid > 0x7fffffffLL || pb.B > 0x7fffffffLL) return -2;
    char* w = (char*)ws;
    uint16_t* Uws = (uint16_t*)(w + pl.off_u);
    uint16_t* dY1ws = (uint16_t*)(w + pl.off_dy1);
    uint16_t* dWws = (uint16_t*)(w + pl.off_dw);
    uint16_t* LT = (uint16_t*)(w + pl.off_lt);
    uint16_t* RT = (uint16_t*)(w + pl.off_rt);
    uint16_t* Rp = (uint16_t*)(w + pl.off_rp);
    const Pack64Job jr{(const uint16_t*)R, Rp, 0}, jlt{(const uint16_t*)L, LT, 1}, jrt{(const uint16_t*)R, RT, 1};
    hipLaunchKernelGGL(pack64_kernel, dim3(3 * 128), dim3(256), 0, st, jr, jlt, jrt);
    hipLaunchKernelGGL(transpose64_kernel, dim3((unsigned)pb.B), dim3(256), 0, st, (const uint16_t*)dy, dWws);
    if (hipGetLastError() != hipSuccess) return -4;
    auto kern = bwd_sq64_data_kernel<false>;
    if (allow_dynamic_lds((const void*)kern, SQ_LDS) != hipSuccess)
        return -4;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), SQ_LDS, st, dWws, (const uint16_t*)x, Rp, LT, RT,
                       (uint16_t*)dx, Uws, dY1ws, pb.B);
    if (hipGetLastError() != hipSuccess) return -4;

    WgradDesc dl, dr;
    fill_descs64(pb, dl, dr);
    dl.A = dWws; dl.Bm = Uws; dl.P = (float*)(w + pl.off_partL); dl.out = dL;
    dr.A = dY1ws; dr.Bm = (const uint16_t*)x; dr.P = (float*)(w + pl.off_partR); dr.out = dR;
    dl.rows_per_chunk = dr.rows_per_chunk = pl.rows_per_chunk;
    dl.p_bf16 = dr.p_bf16 = f32out ? 0 : 1;  // bf16 gradients: bf16 partial tiles
    int rc = wgrad_gemm_pair(dl, dr, pl.nz, st);
    if (rc) return rc;
    return wgrad_reduce_pair(dl, dr, f32out, pl.nz, st);
}

}  // namespace monarch
