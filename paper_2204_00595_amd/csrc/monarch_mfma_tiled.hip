// Shape-generic bf16 matrix-core kernels: the Monarch multiply of Section 3.3 and its backward for
// any number of blocks, with block sizes that are multiples of 16 (forward) or 32 (backward: the tile
// sizes of the weight-gradient GEMMs).  They serve the shapes that have no tuned
// kernel; both readings of the permutation between the factors are handled.
//
// A workgroup (eight waves) owns TB = 16 * RT rows.  A block-diagonal stage is a list of work items
// (block, 16-column output tile) dealt round-robin to the waves; an item keeps RT accumulator tiles
// (one per 16 rows) on v_mfma_f32_16x16x32_bf16, so a weight fragment is loaded once per K-step and
// used RT times.  The vector between the factors lives in LDS only, stored in the order the next
// stage reads it (the permutation is folded into the 2-byte LDS writes of the producing stage), so
// the next stage's operands are 16-byte LDS reads.  A block size that is 16 mod 32 ends on a K-step
// whose upper slots are zero in both operands.
//
// Forward:   step 1 (x, R) -> U in LDS -> step 2 (L) -> y.  A stage-2 item takes CG consecutive blocks
//            c of one 16-row output tile l: y[b][l*k + c] then leaves as CG contiguous values per lane.
// Backward:  dy tile -> LDS as dW[b][c][l] (adjoint of step 3) and to the workspace;
//            step 1 recomputed -> U to the workspace (dL needs it);
//            dU = dW L (per block, weights L^T) -> dY1 order in LDS -> workspace (dR needs it);
//            dx = dY1 R (weights R^T) -> LDS -> full-row stores;
//            dL, dR by the batch-contracted GEMMs of monarch_mfma_wgrad.hip.
#include "monarch_internal.h"
#include "monarch_mfma_common.h"

namespace monarch {

namespace {

constexpr int TL_WAVES = 8, TL_THREADS = 64 * TL_WAVES;
constexpr int KU = 4;  // K-steps (of 32) whose operand loads are in flight together

struct TiledShape {
    int k, p, q, s, perm_b;
};

// Position in U of Y1[kk][j]: the inverse of pi, where U[f] = Y1flat[pi(f)] and
//   default reading:      pi(f) = (f mod k) * q + f / k
//   alternative reading:  pi(f) = (f mod q) * k + f / q
__device__ __forceinline__ int u_of_y1(int kk, int j, const TiledShape& sh)
{
    if (!sh.perm_b) return j * sh.k + kk;
    const int g = kk * sh.q + j;
    return (g % sh.k) * sh.q + g / sh.k;
}
// Position in Y1 (flat) of U[c][r]: pi(c*q + r).
__device__ __forceinline__ int y1_of_u(int c, int r, const TiledShape& sh)
{
    if (sh.perm_b) return r * sh.k + c;
    const int f = c * sh.q + r;
    return (f % sh.k) * sh.q + f / sh.k;
}

__device__ __forceinline__ uint16_t bf16_bits(float v) { return (uint16_t)(pack_bf16x2(v, 0.f) & 0xffffu); }
__device__ __forceinline__ float bf16_value(uint16_t b) { return __builtin_bit_cast(float, (uint32_t)b << 16); }

// One block-diagonal stage:  out[b][blk][n] = sum_i W[blk][n][i] * act[b][blk][i]  for the workgroup's rows.
// load_a(rt, blk, i0) returns the eight activations i0 .. i0+7 of block blk for the lane's row of row tile rt;
// emit(blk, t, acc) receives acc[rt][i] = out[b = 16*rt + 4*(lane/16) + i][blk][16*t + lane%16].
// An item is NT adjacent output tiles of one block: an activation fragment is then loaded once for NT
// weight fragments: the stages are bound by the issue of operand loads, not by the matrix cores.
template <int RT, int NT, typename LoadA, typename Emit>
__device__ __forceinline__ void tiled_stage_nt(int wave, int lane, int nblk, int nout, int nin,
                                               const uint16_t* __restrict__ W, LoadA&& load_a, Emit&& emit)
{
    const int n = lane & 15, kg = lane >> 4;
    const int ntile = (nout >> 4) / NT, items = nblk * ntile;
    const u32x4 zero = {0, 0, 0, 0};
    for (int item = wave; item < items; item += TL_WAVES) {
        const int blk = item / ntile, t = (item - blk * ntile) * NT;
        const uint16_t* wrow = W + ((size_t)blk * nout + 16 * t + n) * nin + 8 * kg;
        f32x4 acc[NT][RT];
#pragma unroll
        for (int j = 0; j < NT; ++j)
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) acc[j][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
        // KU K-steps per round, all of their loads issued before the first MFMA: the waves have nothing else
        // to hide the load latency behind
        for (int k0 = 0; k0 < nin; k0 += 32 * KU) {
            u32x4 wf[KU][NT], af[KU][RT];
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const int i0 = k0 + 32 * u + 8 * kg;
                const bool ok = i0 < nin;
#pragma unroll
                for (int j = 0; j < NT; ++j) wf[u][j] = ok ? ldg128(wrow + (size_t)16 * j * nin + k0 + 32 * u) : zero;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) af[u][rt] = ok ? load_a(rt, blk, i0) : zero;
            }
#pragma unroll
            for (int u = 0; u < KU; ++u)
#pragma unroll
                for (int j = 0; j < NT; ++j)
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt)
                        acc[j][rt] = mfma16(as_bf16x8(af[u][rt]), as_bf16x8(wf[u][j]), acc[j][rt]);
        }
#pragma unroll
        for (int j = 0; j < NT; ++j) emit(blk, t + j, acc[j]);
    }
}

template <int RT, typename LoadA, typename Emit>
__device__ __forceinline__ void tiled_stage(int wave, int lane, int nblk, int nout, int nin,
                                            const uint16_t* __restrict__ W, LoadA&& load_a, Emit&& emit)
{
    // as many tiles per item (at most four) as divide the tile count and still leave every wave an item
    const int ntile = nout >> 4;
    if (ntile % 4 == 0 && nblk * (ntile / 4) >= TL_WAVES)
        tiled_stage_nt<RT, 4>(wave, lane, nblk, nout, nin, W, load_a, emit);
    else if (ntile % 3 == 0 && nblk * (ntile / 3) >= TL_WAVES)
        tiled_stage_nt<RT, 3>(wave, lane, nblk, nout, nin, W, load_a, emit);
    else if (ntile % 2 == 0 && nblk * (ntile / 2) >= TL_WAVES)
        tiled_stage_nt<RT, 2>(wave, lane, nblk, nout, nin, W, load_a, emit);
    else
        tiled_stage_nt<RT, 1>(wave, lane, nblk, nout, nin, W, load_a, emit);
}

// rows x cols LDS tile (row stride ld) -> dst[(b0 + row) * cols + ..] in 16-byte pieces, rows below B only
__device__ __forceinline__ void copy_tile(const uint16_t* T, int ld, int cols, int rows, uint16_t* __restrict__ dst,
                                          int64_t b0, int64_t B, int tid, bool streamed)
{
    const int npc = cols >> 3, total = rows * npc;
    for (int idx = tid; idx < total; idx += TL_THREADS) {
        const int row = idx / npc, pc = idx - row * npc;
        if (b0 + row >= B) break;  // rows grow with idx
        const u32x4 v = lds128(T + (size_t)row * ld + 8 * pc);
        uint16_t* p = dst + (size_t)(b0 + row) * cols + 8 * pc;
        if (streamed) stg128_nt(p, v);
        else *reinterpret_cast<u32x4*>(p) = v;
    }
}

template <int N>
__device__ __forceinline__ void store_run(uint16_t* p, const float (&v)[N])
{
    if constexpr (N == 8) {
        *reinterpret_cast<u32x4*>(p) =
            u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
    } else if constexpr (N == 4) {
        *reinterpret_cast<u32x2*>(p) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
    } else if constexpr (N == 2) {
        *reinterpret_cast<uint32_t*>(p) = pack_bf16x2(v[0], v[1]);
    } else {
        *p = bf16_bits(v[0]);
    }
}

// ---------------------------------------------------------------------------- forward ----

// Second stage of the forward for the workgroup's rows: y[b][l*k + c] = sum_r L[c][l][r] * U[b][c*q + r] (+ bias),
// U in LDS (row stride ldu).
template <int RT, int CG, int NL>
__device__ __forceinline__ void fwd_stage2(int wave, int lane, const uint16_t* __restrict__ L, const uint16_t* lds, int ldu,
                                           uint16_t* __restrict__ y, const uint16_t* __restrict__ bias, int64_t b0,
                                           int64_t B, const TiledShape& sh)
{
    const int m = lane & 15, kg = lane >> 4;
    const int n_out = sh.k * sh.s;
    constexpr int KU2 = CG * NL >= 8 ? 2 : KU;  // many accumulators: fewer K-steps in flight, or they spill
    const int ncg = sh.k / CG, items = ((sh.s >> 4) / NL) * ncg;
    const u32x4 zero = {0, 0, 0, 0};
    for (int item = wave; item < items; item += TL_WAVES) {
        const int lt = (item / ncg) * NL, cgi = item % ncg;
        f32x4 acc[CG][NL][RT];
#pragma unroll
        for (int cc = 0; cc < CG; ++cc)
#pragma unroll
            for (int j = 0; j < NL; ++j)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) acc[cc][j][rt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < CG; ++cc) {
            const int c = cgi * CG + cc;
            const uint16_t* wrow = L + ((size_t)c * sh.s + 16 * lt + m) * sh.q + 8 * kg;
            const uint16_t* urow = lds + (size_t)m * ldu + c * sh.q + 8 * kg;
            for (int k0 = 0; k0 < sh.q; k0 += 32 * KU2) {
                u32x4 wf[KU2][NL], af[KU2][RT];
#pragma unroll
                for (int u = 0; u < KU2; ++u) {
                    const bool ok = k0 + 32 * u + 8 * kg < sh.q;
#pragma unroll
                    for (int j = 0; j < NL; ++j) wf[u][j] = ok ? ldg128(wrow + (size_t)16 * j * sh.q + k0 + 32 * u) : zero;
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) af[u][rt] = ok ? lds128(urow + (size_t)16 * rt * ldu + k0 + 32 * u) : zero;
                }
#pragma unroll
                for (int u = 0; u < KU2; ++u)
#pragma unroll
                    for (int j = 0; j < NL; ++j)
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt)
                            acc[cc][j][rt] = mfma16(as_bf16x8(af[u][rt]), as_bf16x8(wf[u][j]), acc[cc][j][rt]);
            }
        }
        // the lane holds output index l = 16*(lt + j) + m of blocks c0 .. c0+CG-1: columns l*k + c0 .. are contiguous
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const int col = (16 * (lt + j) + m) * sh.k + cgi * CG;
            float bv[CG];
#pragma unroll
            for (int cc = 0; cc < CG; ++cc) bv[cc] = bias ? bf16_value(bias[col + cc]) : 0.f;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int64_t row = b0 + 16 * rt + 4 * kg + i;
                    if (row < B) {
                        float v[CG];
#pragma unroll
                        for (int cc = 0; cc < CG; ++cc) v[cc] = acc[cc][j][rt][i] + bv[cc];
                        store_run<CG>(y + (size_t)row * n_out + col, v);
                    }
                }
        }
    }
}

template <int RT, int CG>
__global__ void __launch_bounds__(TL_THREADS)
tiled_fwd_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ R, const uint16_t* __restrict__ L,
                 uint16_t* __restrict__ y, const uint16_t* __restrict__ bias, int64_t B, TiledShape sh, int ldu)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];  // U[TB][ldu]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, m = lane & 15, kg = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * (16 * RT);
    const int n_in = sh.k * sh.p;

    // rows past the end are computed from the last valid row and dropped at the store
    const uint16_t* xrow[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        int64_t r = b0 + 16 * rt + m;
        r = r < B ? r : B - 1;
        xrow[rt] = x + (size_t)r * n_in;
    }
    tiled_stage<RT>(
        wave, lane, sh.k, sh.q, sh.p, R, [&](int rt, int blk, int i0) { return ldg128(xrow[rt] + blk * sh.p + i0); },
        [&](int kk, int t, const f32x4(&acc)[RT]) {
            const int f = u_of_y1(kk, 16 * t + m, sh);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int i = 0; i < 4; ++i) lds[(size_t)(16 * rt + 4 * kg + i) * ldu + f] = bf16_bits(acc[rt][i]);
        });
    __syncthreads();

    // An item: CG consecutive blocks c of NL adjacent 16-row output tiles l.  NL = 2 (an activation fragment
    // from LDS then serves two weight fragments) where the accumulators fit and every wave still gets an item.
    const int ltiles = sh.s >> 4, ncg = sh.k / CG;
    if (CG <= 4 && (ltiles & 1) == 0 && (ltiles >> 1) * ncg >= TL_WAVES)
        fwd_stage2<RT, CG, 2>(wave, lane, L, lds, ldu, y, bias, b0, B, sh);
    else
        fwd_stage2<RT, CG, 1>(wave, lane, L, lds, ldu, y, bias, b0, B, sh);
}

// ---------------------------------------------------------------------------- backward ----

// dst[blk][c][r] = src[blk][r][c] for the blocks of both factors (blockIdx.y picks the factor)
struct TransposeJob {
    const uint16_t* src;
    uint16_t* dst;
    int nblk, rows, cols;
};
__global__ void __launch_bounds__(256) transpose_blocks_kernel(TransposeJob j0, TransposeJob j1)
{
    const TransposeJob& j = blockIdx.y == 0 ? j0 : j1;
    const size_t per = (size_t)j.rows * j.cols, total = per * j.nblk;
    const size_t o = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (o >= total) return;
    const size_t blk = o / per, rem = o - blk * per;
    const int c = (int)(rem / j.rows), r = (int)(rem - (size_t)c * j.rows);
    j.dst[o] = j.src[blk * per + (size_t)r * j.cols + c];
}

// DX_ONLY: the transposed multiply y = x M on its own (dy is then its input, dx its output): no recompute
// of step 1, no workspace copies.
template <int RT, bool DX_ONLY>
__global__ void __launch_bounds__(TL_THREADS)
tiled_bwd_kernel(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ x, const uint16_t* __restrict__ R,
                 const uint16_t* __restrict__ LT /* [c][r][l] */, const uint16_t* __restrict__ RTr /* [kk][i][j] */,
                 uint16_t* __restrict__ dx, uint16_t* __restrict__ Uws, uint16_t* __restrict__ dWws,
                 uint16_t* __restrict__ dY1ws, int64_t B, TiledShape sh, int ld1, int ldu)
{
    constexpr int TB = 16 * RT;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* T1 = lds;                     // [TB][ld1]: dW tile, later the dx tile
    uint16_t* T2 = lds + (size_t)TB * ld1;  // [TB][ldu]: U tile, later the dY1 tile
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, m = lane & 15, kg = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * TB;
    const int n_in = sh.k * sh.p, n_out = sh.k * sh.s, kq = sh.k * sh.q;

    // ---- adjoint of step 3: dW[b][c][l] = dy[b][l*k + c], de-interleaved into T1
    {
        const int npc = n_out >> 3, total = TB * npc;
        for (int idx = tid; idx < total; idx += TL_THREADS) {
            const int row = idx / npc, pc = idx - row * npc;
            int64_t r = b0 + row;
            r = r < B ? r : B - 1;
            const u32x4 v = ldg128(dy + (size_t)r * n_out + 8 * pc);
            int l = (8 * pc) / sh.k, c = (8 * pc) - l * sh.k;
            uint16_t* trow = T1 + (size_t)row * ld1;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t w = v[e >> 1];
                trow[c * sh.s + l] = (uint16_t)((e & 1) ? (w >> 16) : (w & 0xffffu));
                if (++c == sh.k) {
                    c = 0;
                    ++l;
                }
            }
        }
    }

    // ---- step 1 again: U to T2, in stage-2 order
    if constexpr (!DX_ONLY) {
        const uint16_t* xrow[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            int64_t r = b0 + 16 * rt + m;
            r = r < B ? r : B - 1;
            xrow[rt] = x + (size_t)r * n_in;
        }
        tiled_stage<RT>(
            wave, lane, sh.k, sh.q, sh.p, R, [&](int rt, int blk, int i0) { return ldg128(xrow[rt] + blk * sh.p + i0); },
            [&](int kk, int t, const f32x4(&acc)[RT]) {
                const int f = u_of_y1(kk, 16 * t + m, sh);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) T2[(size_t)(16 * rt + 4 * kg + i) * ldu + f] = bf16_bits(acc[rt][i]);
            });
    }
    __syncthreads();
    if constexpr (!DX_ONLY) {
        copy_tile(T2, ldu, kq, TB, Uws, b0, B, tid, false);
        copy_tile(T1, ld1, n_out, TB, dWws, b0, B, tid, false);
        __syncthreads();  // U has left T2
    }

    // ---- adjoint of step 2: dU[b][c][r] = sum_l L[c][l][r] dW[b][c][l], written where dY1 has it
    tiled_stage<RT>(
        wave, lane, sh.k, sh.q, sh.s, LT,
        [&](int rt, int blk, int i0) { return lds128(T1 + (size_t)(16 * rt + m) * ld1 + blk * sh.s + i0); },
        [&](int c, int t, const f32x4(&acc)[RT]) {
            const int g = y1_of_u(c, 16 * t + m, sh);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int i = 0; i < 4; ++i) T2[(size_t)(16 * rt + 4 * kg + i) * ldu + g] = bf16_bits(acc[rt][i]);
        });
    __syncthreads();  // dY1 complete; nobody reads dW any more
    if constexpr (!DX_ONLY) copy_tile(T2, ldu, kq, TB, dY1ws, b0, B, tid, false);

    // ---- adjoint of step 1: dx[b][kk*p + i] = sum_j R[kk][j][i] dY1[b][kk][j], staged in T1
    tiled_stage<RT>(
        wave, lane, sh.k, sh.p, sh.q, RTr,
        [&](int rt, int blk, int i0) { return lds128(T2 + (size_t)(16 * rt + m) * ldu + blk * sh.q + i0); },
        [&](int kk, int t, const f32x4(&acc)[RT]) {
            const int col = kk * sh.p + 16 * t + m;
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int i = 0; i < 4; ++i) T1[(size_t)(16 * rt + 4 * kg + i) * ld1 + col] = bf16_bits(acc[rt][i]);
        });
    __syncthreads();
    copy_tile(T1, ld1, n_in, TB, dx, b0, B, tid, true);
}

// ---------------------------------------------------------------------------- host ----

// Row tiles per workgroup: the most whose LDS tile fits (every workgroup streams all the weights through
// its L1 once, so fewer, larger tiles win over more resident workgroups); not more rows than the batch has.
// 0: does not fit.
int pick_rt(size_t row_bytes, int64_t B)
{
    int rt = 0;
    for (int c : {4, 2, 1})
        if ((size_t)16 * c * row_bytes <= kMaxLdsBytes) {
            rt = c;
            break;
        }
    while (rt > 1 && (int64_t)16 * (rt / 2) >= B) rt /= 2;
    return rt;
}

bool base_ok(const Problem& pb)
{
    return pb.dtype == 1 && pb.p % 16 == 0 && pb.q % 16 == 0 && pb.s % 16 == 0;
}

size_t fwd_row_bytes(const Problem& pb) { return ((size_t)pb.kq() + 8) * 2; }
int bwd_ld1(const Problem& pb) { return (pb.n_out() > pb.n_in ? pb.n_out() : pb.n_in) + 8; }
size_t bwd_row_bytes(const Problem& pb) { return ((size_t)bwd_ld1(pb) + pb.kq() + 8) * 2; }

TiledShape shape_of(const Problem& pb) { return TiledShape{pb.k, pb.p, pb.q, pb.s, pb.perm_b() ? 1 : 0}; }

template <int RT, int CG>
int launch_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    const int ldu = pb.kq() + 8;
    const size_t lds = (size_t)16 * RT * ldu * 2;
    auto kern = tiled_fwd_kernel<RT, CG>;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    const int64_t grid = (pb.B + 16 * RT - 1) / (16 * RT);
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(TL_THREADS), lds, st, (const uint16_t*)x, (const uint16_t*)R,
                       (const uint16_t*)L, (uint16_t*)y, (const uint16_t*)pb.bias, pb.B, shape_of(pb), ldu);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Blocks per stage-2 item: the most that divide k.  (Fewer blocks per item would deal the items more
// evenly to the waves, e.g. 24 instead of 6 for s = 96, k = 4, but the narrower stores cost more: 18.7 vs 17.3 us.)
int pick_cg(const Problem& pb)
{
    for (int c : {8, 4, 2})
        if (pb.k % c == 0) return c;
    return 1;
}

template <int RT>
int launch_fwd_cg(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    switch (pick_cg(pb)) {
        case 8: return launch_fwd<RT, 8>(pb, x, R, L, y, st);
        case 4: return launch_fwd<RT, 4>(pb, x, R, L, y, st);
        case 2: return launch_fwd<RT, 2>(pb, x, R, L, y, st);
    }
    return launch_fwd<RT, 1>(pb, x, R, L, y, st);
}

// Workspace of the backward: the three row-major intermediates, the transposed factors, the partial
// tiles of the two weight-gradient GEMMs (nz batch chunks: about one workgroup per CU).
struct TiledPlan {
    size_t off_u, off_dw, off_dy1, off_lt, off_rt, off_partL, off_partR, total;
    int nz, rows_per_chunk;
    bool ok;
};

void fill_descs_tiled(const Problem& pb, WgradDesc& dl, WgradDesc& dr)
{
    // dL[c][l][r] = sum_b dW[b][c][l] * U[b][c*q + r]
    dl = WgradDesc{};
    dl.lda = pb.n_out(); dl.a_g = pb.s; dl.deint = 0;
    dl.ldb = pb.kq(); dl.b_g = pb.q; dl.b_seg = 0; dl.seg_w = pb.q;
    dl.M = pb.s; dl.N = pb.q; dl.G = pb.k; dl.rows = pb.B;
    // dR[kk][j][i] = sum_b dY1[b][kk][j] * x[b][kk*p + i]
    dr = WgradDesc{};
    dr.lda = pb.kq(); dr.a_g = pb.q; dr.deint = 0;
    dr.ldb = pb.n_in; dr.b_g = pb.p; dr.b_seg = 0; dr.seg_w = pb.p;
    dr.M = pb.q; dr.N = pb.p; dr.G = pb.k; dr.rows = pb.B;
}

TiledPlan make_plan_tiled(const Problem& pb)
{
    TiledPlan pl{};
    WgradDesc dl, dr;
    fill_descs_tiled(pb, dl, dr);
    const int tl = wgrad_tiles(dl), tr = wgrad_tiles(dr);
    pl.ok = tl > 0 && tr > 0;
    if (!pl.ok) return pl;
    int64_t z = 256 / (tl + tr);
    const int64_t maxz = (pb.B + 255) / 256;
    if (z > maxz) z = maxz;
    if (z < 1) z = 1;
    const int64_t rpc = ((pb.B + z - 1) / z + 63) / 64 * 64;
    pl.rows_per_chunk = (int)(rpc > 0 ? rpc : 64);
    pl.nz = (int)((pb.B + pl.rows_per_chunk - 1) / pl.rows_per_chunk);
    if (pl.nz < 1) pl.nz = 1;
    const size_t rows = (size_t)(pb.B > 0 ? pb.B : 1);
    size_t off = 0;
    pl.off_u = off;   off += align_up(rows * pb.kq() * 2, 256);
    pl.off_dw = off;  off += align_up(rows * pb.n_out() * 2, 256);
    pl.off_dy1 = off; off += align_up(rows * pb.kq() * 2, 256);
    pl.off_lt = off;  off += align_up(pb.n_L() * 2, 256);
    pl.off_rt = off;  off += align_up(pb.n_R() * 2, 256);
    pl.off_partL = off; off += align_up((size_t)pl.nz * pb.n_L() * 4, 256);
    pl.off_partR = off; off += align_up((size_t)pl.nz * pb.n_R() * 4, 256);
    pl.total = off;
    return pl;
}

template <int RT, bool DX_ONLY>
int launch_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const uint16_t* LT, const uint16_t* RTr,
               void* dx, uint16_t* Uws, uint16_t* dWws, uint16_t* dY1ws, hipStream_t st)
{
    const int ld1 = bwd_ld1(pb), ldu = pb.kq() + 8;
    const size_t lds = (size_t)16 * RT * (ld1 + ldu) * 2;
    auto kern = tiled_bwd_kernel<RT, DX_ONLY>;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    const int64_t grid = (pb.B + 16 * RT - 1) / (16 * RT);
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(TL_THREADS), lds, st, (const uint16_t*)dy, (const uint16_t*)x,
                       (const uint16_t*)R, LT, RTr, (uint16_t*)dx, Uws, dWws, dY1ws, pb.B, shape_of(pb), ld1, ldu);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

template <bool DX_ONLY>
int launch_bwd_rt(const Problem& pb, const void* dy, const void* x, const void* R, const uint16_t* LT, const uint16_t* RTr,
                  void* dx, uint16_t* Uws, uint16_t* dWws, uint16_t* dY1ws, hipStream_t st)
{
    switch (pick_rt(bwd_row_bytes(pb), pb.B)) {
        case 4: return launch_bwd<4, DX_ONLY>(pb, dy, x, R, LT, RTr, dx, Uws, dWws, dY1ws, st);
        case 2: return launch_bwd<2, DX_ONLY>(pb, dy, x, R, LT, RTr, dx, Uws, dWws, dY1ws, st);
        case 1: return launch_bwd<1, DX_ONLY>(pb, dy, x, R, LT, RTr, dx, Uws, dWws, dY1ws, st);
    }
    return -2;
}

// L^T and R^T (per block) into the workspace
int launch_transposes(const Problem& pb, const void* R, const void* L, uint16_t* LT, uint16_t* RTr, hipStream_t st)
{
    const TransposeJob jl{(const uint16_t*)L, LT, pb.k, pb.s, pb.q};
    const TransposeJob jr{(const uint16_t*)R, RTr, pb.k, pb.q, pb.p};
    const size_t nmax = pb.n_L() > pb.n_R() ? pb.n_L() : pb.n_R();
    hipLaunchKernelGGL(transpose_blocks_kernel, dim3((unsigned)((nmax + 255) / 256), 2), dim3(256), 0, st, jl, jr);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // namespace

bool tiled_fwd_supported(const Problem& pb) { return base_ok(pb) && pick_rt(fwd_row_bytes(pb), pb.B > 0 ? pb.B : 1) > 0; }

int tiled_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if (!tiled_fwd_supported(pb)) return -2;
    switch (pick_rt(fwd_row_bytes(pb), pb.B)) {
        case 4: return launch_fwd_cg<4>(pb, x, R, L, y, st);
        case 2: return launch_fwd_cg<2>(pb, x, R, L, y, st);
        case 1: return launch_fwd_cg<1>(pb, x, R, L, y, st);
    }
    return -2;
}

bool tiled_bwd_supported(const Problem& pb)
{
    return base_ok(pb) && pb.p % 32 == 0 && pb.q % 32 == 0 && pb.s % 32 == 0 &&
           pick_rt(bwd_row_bytes(pb), pb.B > 0 ? pb.B : 1) > 0 && make_plan_tiled(pb).ok;
}

size_t tiled_bwd_workspace(const Problem& pb) { return make_plan_tiled(pb).total; }

int tiled_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
              void* dL, void* ws, hipStream_t st)
{
    if (!tiled_bwd_supported(pb)) return -2;
    const TiledPlan pl = make_plan_tiled(pb);
    const bool f32out = pb.wgrad_f32();
    if (pb.B == 0) {
        int rc = f32out ? launch_fill_zero_f32((float*)dR, pb.n_R(), st) : launch_fill_zero_u16((uint16_t*)dR, pb.n_R(), st);
        if (rc) return rc;
        return f32out ? launch_fill_zero_f32((float*)dL, pb.n_L(), st) : launch_fill_zero_u16((uint16_t*)dL, pb.n_L(), st);
    }
    char* w = (char*)ws;
    uint16_t* LT = (uint16_t*)(w + pl.off_lt);
    uint16_t* RTr = (uint16_t*)(w + pl.off_rt);
    int rc = launch_transposes(pb, R, L, LT, RTr, st);
    if (rc) return rc;
    rc = launch_bwd_rt<false>(pb, dy, x, R, LT, RTr, dx, (uint16_t*)(w + pl.off_u), (uint16_t*)(w + pl.off_dw),
                              (uint16_t*)(w + pl.off_dy1), st);
    if (rc) return rc;
    WgradDesc dl, dr;
    fill_descs_tiled(pb, dl, dr);
    dl.A = (const uint16_t*)(w + pl.off_dw); dl.Bm = (const uint16_t*)(w + pl.off_u);
    dl.P = (float*)(w + pl.off_partL); dl.out = dL;
    dr.A = (const uint16_t*)(w + pl.off_dy1); dr.Bm = (const uint16_t*)x;
    dr.P = (float*)(w + pl.off_partR); dr.out = dR;
    dl.rows_per_chunk = dr.rows_per_chunk = pl.rows_per_chunk;
    dl.p_bf16 = dr.p_bf16 = f32out ? 0 : 1;  // bf16 gradients: bf16 partial tiles
    rc = wgrad_gemm_pair(dl, dr, pl.nz, st);
    if (rc) return rc;
    return wgrad_reduce_pair(dl, dr, f32out, pl.nz, st);
}

// Transposed multiply y = x M (input rows of k*s values, output rows of n_in): the two adjoint stages alone.
bool tiled_fwd_t_supported(const Problem& pb) { return base_ok(pb) && pick_rt(bwd_row_bytes(pb), pb.B > 0 ? pb.B : 1) > 0; }
size_t tiled_fwd_t_workspace(const Problem& pb) { return align_up(pb.n_L() * 2, 256) + align_up(pb.n_R() * 2, 256); }
int tiled_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    if (!tiled_fwd_t_supported(pb)) return -2;
    uint16_t* LT = (uint16_t*)ws;
    uint16_t* RTr = (uint16_t*)((char*)ws + align_up(pb.n_L() * 2, 256));
    const int rc = launch_transposes(pb, R, L, LT, RTr, st);
    if (rc) return rc;
    return launch_bwd_rt<true>(pb, x, nullptr, R, LT, RTr, y, nullptr, nullptr, nullptr, st);
}

}  // namespace monarch
