// Weight gradients of the Monarch multiply as batched "TN" GEMMs on bf16 MFMA:
//
//     out[g][m][n] = sum_b  A[b][g, m] * Bm[b][g, n]            (contraction over the batch)
//
//   dL[c][l][r]  = sum_b dW[b][c][l] * U[b][c*q + r]     A = dy (column l*k + c),  Bm = U
//   dR[kk][j][i] = sum_b dY1[b][kk][j] * x[b][kk*p + i]  A = dY1,                  Bm = x
//
// (the adjoints of steps 2 and 1 of Section 3.3).  Both operands are stored batch-major, i.e.
// the contraction index is the slow one, so they are staged row-major in LDS with 16-byte
// writes and read back with the transposing LDS load of gfx950 (ds_read_b64_tr_b16), which
// hands every lane four consecutive batch rows of one feature: exactly the MFMA operand layout.
//
// One workgroup = four groups g, two waves per group (each takes every other 16-row K-step on its own
// accumulators: two waves per SIMD hide each other's staging and LDS latencies), a TM x TN tile of
// each group's output; the batch is split into chunks whose fp32 partial tiles are summed by
// `wgrad_reduce_kernel`, which also undoes the column order used for dL and converts to the
// output type.
#include "monarch_internal.h"
#include "monarch_mfma_common.h"
#include "monarch_colsum.h"

namespace monarch {

namespace {

typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int KB = 32;    // batch rows per pipeline step (two 16-row K-steps, one per wave of a group)
constexpr int NTHR = 512;  // eight waves per workgroup
constexpr int NSTG = 1;     // register stages of the operand loads (rows fetched NSTG steps before they are stored)

// Padding of the LDS rows (bf16 elements).  A half wave of a transposing read touches four consecutive rows,
// 64 bytes (16 banks) of each: with a row stride of an odd multiple of 64 bytes the four rows fall on disjoint
// quarters of the 64 banks.  Strides: 128 -> 160, 96 -> 96, 64 -> 96, 32 -> 32 elements.  (The 16-byte writes stay
// conflict-free: 16 lanes write 256 bytes that are either contiguous or in two disjoint bank ranges.)
constexpr int lds_pad(int tile) { return (tile == 128 || tile == 64) ? 32 : 0; }

// Transposing LDS read: within each 16 lanes, lane i receives element (i % 4) of lanes
// i/4, 4 + i/4, 8 + i/4, 12 + i/4.
__device__ __forceinline__ u32x2 lds_tr16(const uint16_t* p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(const_cast<uint16_t*>(p)));
    return __builtin_bit_cast(u32x2, v);
}

// MFMA operand (32 features x 16 batch rows) from a row-major LDS tile T[row][col]:
// lane (f = lane % 32, h = lane / 32) gets T[k0 + 8h .. 8h+7][c0 + f].
__device__ __forceinline__ bf16x8 frag_tr(const uint16_t* T, int stride, int k0, int c0, int lane)
{
    const int G = lane >> 4, j = lane & 15;
    const uint16_t* p = T + (size_t)(k0 + 8 * (G >> 1) + (j >> 2)) * stride + c0 + 16 * (G & 1) + 4 * (j & 3);
    const u32x2 lo = lds_tr16(p), hi = lds_tr16(p + 4 * stride);
    const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
    return as_bf16x8(v);
}

// MSPLIT = false: the two waves of a group split the K-steps (each keeps the whole TM x TN tile, summed at the end);
// MSPLIT = true (large tiles): they split the tile's rows m instead, each taking both K-steps of a pipeline step on
// its own half of the accumulators -- 128 x 128 per group in 2 x 128 accumulator registers, which halves the operand
// bytes fetched per flop against the 64 x 128 tile.
template <int TM, int TN, bool DEINT, bool MSPLIT>
__device__ __forceinline__ void wgrad_gemm_body(const WgradDesc& d, const int tile, const int zi)
{
    constexpr int MT = TM / 32, NT = TN / 32;
    constexpr int MTW = MSPLIT ? MT / 2 : MT;  // m tiles of one wave
    static_assert(!MSPLIT || MT % 2 == 0, "row split");
    constexpr int SA = TM + lds_pad(TM), SB = TN + lds_pad(TN);  // LDS row strides (bf16 elements)
    constexpr int BUF = 4 * KB * (SA + SB);  // one pipeline buffer: As [4][KB][SA], then Bs [4][KB][SB]
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];

    // eight waves: wave = (group g, half kh); the two waves of a group each take one 16-row K-step of every
    // 32-row pipeline step on their own accumulators, which are summed through LDS at the end (MSPLIT: each
    // takes half of the tile's rows m over both K-steps, and nothing is summed)
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int grp = wave & 3, kh = wave >> 2;
    const int tiles_n = d.N / TN;
    const int tiles_mn = (d.M / TM) * tiles_n;
    const int g0 = (tile / tiles_mn) * 4, tmn = tile % tiles_mn;
    const int m0 = (tmn / tiles_n) * TM, n0 = (tmn % tiles_n) * TN;
    const int64_t row_lo = (int64_t)zi * d.rows_per_chunk;
    int64_t row_hi = row_lo + d.rows_per_chunk;
    if (row_hi > d.rows) row_hi = d.rows;
    const int64_t nrows = row_hi > row_lo ? row_hi - row_lo : 0;

    // ---- per-thread load tasks (16-byte pieces; DEINT A: 64-byte runs holding 8 m x 4 groups) ----
    // Addresses are fixed for the whole chunk: global pointers at row_lo (advanced by a uniform row
    // offset per step), LDS offsets inside a buffer, and the row of the task inside a step.
    constexpr int A_TASKS = DEINT ? (KB * TM / 8) : (4 * KB * TM / 8);
    constexpr int B_TASKS = 4 * KB * TN / 8;
    constexpr int A_PER = (A_TASKS + NTHR - 1) / NTHR, B_PER = (B_TASKS + NTHR - 1) / NTHR;
    u32x4 areg[NSTG][A_PER][DEINT ? 4 : 1], breg[NSTG][B_PER];
    const uint16_t* pa[A_PER];
    const uint16_t* pb[B_PER];
    int ra[A_PER], rb[B_PER], la[A_PER], lb[B_PER];
#pragma unroll
    for (int t = 0; t < A_PER; ++t) {
        // a thread without a task in this slot repeats task 0 (its loads are unconditional and must
        // stay in bounds; it stores nothing)
        const int task = tid + t * NTHR < A_TASKS ? tid + t * NTHR : 0;
        if (DEINT) {
            const int r = task / (TM / 8), u = task % (TM / 8);
            ra[t] = tid + t * NTHR < A_TASKS ? r : (1 << 30);
            pa[t] = d.A + (row_lo + r) * d.lda + (size_t)(m0 + 8 * u) * 4 + g0;
            la[t] = r * SA + 8 * u;
        } else {
            const int g = task / (KB * TM / 8), rem = task % (KB * TM / 8);
            const int r = rem / (TM / 8), u = rem % (TM / 8);
            ra[t] = tid + t * NTHR < A_TASKS && g0 + g < d.G ? r : (1 << 30);  // a group past the last one: zeros
            pa[t] = d.A + (row_lo + r) * d.lda + (size_t)(g0 + g) * d.a_g + m0 + 8 * u;
            la[t] = (g * KB + r) * SA + 8 * u;
        }
    }
#pragma unroll
    for (int t = 0; t < B_PER; ++t) {
        const int task = tid + t * NTHR < B_TASKS ? tid + t * NTHR : 0;
        const int g = task / (KB * TN / 8), rem = task % (KB * TN / 8);
        const int r = rem / (TN / 8), u = rem % (TN / 8);
        const int n = n0 + 8 * u;
        rb[t] = tid + t * NTHR < B_TASKS && g0 + g < d.G ? r : (1 << 30);
        pb[t] = d.Bm + (row_lo + r) * d.ldb + (size_t)(g0 + g) * d.b_g + (size_t)(n / d.seg_w) * d.b_seg + (n % d.seg_w);
        lb[t] = 4 * KB * SA + (g * KB + r) * SB + 8 * u;
    }

    // rows r0 .. r0+KB-1 of the chunk -> register stage `stg`; rows past the end of the chunk (and the
    // slots of threads without a task) load nothing and read as zeros.  (Unconditional loads of a
    // clamped row with the zeroing moved to store_step were measured 10 % slower.)
    auto load_step = [&](int64_t r0, int stg) {
        const int64_t oa = r0 * d.lda, ob = r0 * d.ldb;
#pragma unroll
        for (int t = 0; t < A_PER; ++t) {
            const bool ok = r0 + ra[t] < nrows;
            const uint16_t* p = pa[t] + oa;
#pragma unroll
            for (int w = 0; w < (DEINT ? 4 : 1); ++w) areg[stg][t][w] = ok ? ldg128(p + 8 * w) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int t = 0; t < B_PER; ++t) {
            const bool ok = r0 + rb[t] < nrows;
            breg[stg][t] = ok ? ldg128(pb[t] + ob) : u32x4{0, 0, 0, 0};
        }
    };
    // register stage -> LDS buffer
    auto store_step = [&](int64_t, int stg, uint16_t* buf) {
#pragma unroll
        for (int t = 0; t < A_PER; ++t) {
            if (ra[t] >= KB) continue;
            if (DEINT) {
                // the run holds elements e = 4*m' + c (m' = 0..7); gather the 8 m' of each group c
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    u32x4 v;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const uint32_t lo = areg[stg][t][w][c >> 1], hi = areg[stg][t][w][2 + (c >> 1)];
                        v[w] = (c & 1) ? pick_hi16(lo, hi) : pick_lo16(lo, hi);
                    }
                    *reinterpret_cast<u32x4*>(buf + c * KB * SA + la[t]) = v;
                }
            } else {
                *reinterpret_cast<u32x4*>(buf + la[t]) = areg[stg][t][0];
            }
        }
#pragma unroll
        for (int t = 0; t < B_PER; ++t) {
            if (rb[t] >= KB) continue;
            *reinterpret_cast<u32x4*>(buf + lb[t]) = breg[stg][t];
        }
    };

    f32x16 acc[MTW * NT];
#pragma unroll
    for (int t = 0; t < MTW * NT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    // Pipeline (one workgroup barrier per 32-row step, two LDS buffers, one register stage):
    // in step s the MFMAs read buffer s%2 while the rows of step s+1 go from registers to buffer
    // (s+1)%2 and the rows of step s+2 are fetched into the registers just freed.  A wave reads the
    // fragments of its own K-step (rows 16*kh .. 16*kh+15 of the step) before the staging work, so that
    // their LDS latency hides behind it.  The loop body has no branches (a step past the end of the
    // chunk works on zeros): control flow here makes the compiler shuffle the accumulators between blocks.
    if (nrows > 0) {  // (uniform) an empty chunk touches no memory and yields a zero partial tile
    load_step(0, 0);
    store_step(0, 0, lds);
    load_step(KB, 0);
    const int woff_a = grp * KB * SA, woff_b = 4 * KB * SA + grp * KB * SB;
    for (int64_t r0 = 0; r0 < nrows; r0 += 2 * KB) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const uint16_t* cur = lds + k * BUF;
            uint16_t* nxt = lds + (k ^ 1) * BUF;
            __syncthreads();
            bf16x8 af[MTW], bfr[NT];
            const int krow = MSPLIT ? 0 : 16 * kh, mcol = MSPLIT ? kh * MTW * 32 : 0;
            if constexpr (MSPLIT) {
                // large tiles: the next rows are requested first, so that they travel during the fragment reads too
                store_step(r0 + (k + 1) * KB, 0, nxt);
                load_step(r0 + (k + 2) * KB, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt) af[mt] = frag_tr(cur + woff_a, SA, krow, mcol + mt * 32, lane);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bfr[nt] = frag_tr(cur + woff_b, SB, krow, nt * 32, lane);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!MSPLIT) {
                store_step(r0 + (k + 1) * KB, 0, nxt);
                load_step(r0 + (k + 2) * KB, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[mt * NT + nt] = mfma32(af[mt], bfr[nt], acc[mt * NT + nt]);
            if constexpr (MSPLIT) {
                // second K-step of the pipeline step (rows 16 .. 31 of the buffer)
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt) af[mt] = frag_tr(cur + woff_a, SA, 16, mcol + mt * 32, lane);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bfr[nt] = frag_tr(cur + woff_b, SB, 16, nt * 32, lane);
#pragma unroll
                for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) acc[mt * NT + nt] = mfma32(af[mt], bfr[nt], acc[mt * NT + nt]);
            }
        }
    }
    }

    // sum the two K halves of every group through LDS (fp32, in two rounds of at most R1 tiles per
    // wave: the staging buffers hold 4 x R1 tiles), then the kh = 0 wave owns the group's partial tile
    if constexpr (!MSPLIT) {
        constexpr int NTILE = MT * NT, R1 = (NTILE + 1) / 2;
        static_assert((size_t)4 * R1 * 4096 <= (size_t)2 * BUF * 2, "reduction staging fits the pipeline buffers");
        float* red = reinterpret_cast<float*>(lds) + (size_t)grp * R1 * 1024 + lane;
#pragma unroll
        for (int t0 = 0; t0 < NTILE; t0 += R1) {
            __syncthreads();  // the buffers (or the previous round) are no longer read
            if (kh == 1) {
#pragma unroll
                for (int t = t0; t < t0 + R1 && t < NTILE; ++t)
#pragma unroll
                    for (int i = 0; i < 16; ++i) red[(t - t0) * 1024 + i * 64] = acc[t][i];
            }
            __syncthreads();
            if (kh == 0) {
#pragma unroll
                for (int t = t0; t < t0 + R1 && t < NTILE; ++t)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[t][i] += red[(t - t0) * 1024 + i * 64];
            }
        }
        if (kh != 0) return;
    }
    if (g0 + grp >= d.G) return;  // (the group count need not be a multiple of four)

    // partial tile: P[z][g][m][n]
    const int ln = lane & 31, h = lane >> 5;
    const int mw = m0 + (MSPLIT ? kh * MTW * 32 : 0);  // first row of this wave's accumulators
    const size_t pbase = (((size_t)zi * d.G + g0 + grp) * d.M) * d.N;
    if (d.p_bf16) {
        uint16_t* Pg = reinterpret_cast<uint16_t*>(d.P) + pbase;
#pragma unroll
        for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int m = mw + mt * 32 + 8 * (i / 4) + 4 * h + (i % 4);
                    Pg[(size_t)m * d.N + n0 + nt * 32 + ln] = (uint16_t)(pack_bf16x2(acc[mt * NT + nt][i], 0.f) & 0xffffu);
                }
        return;
    }
    float* Pg = d.P + pbase;
#pragma unroll
    for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int m = mw + mt * 32 + 8 * (i / 4) + 4 * h + (i % 4);
                Pg[(size_t)m * d.N + n0 + nt * 32 + ln] = acc[mt * NT + nt][i];
            }
}

// One launch for up to two GEMMs over the same batch chunks.  Workgroups are handed to the
// eight XCDs round-robin by linear id; the id is remapped so that each XCD owns a contiguous
// range of (chunk, tile) pairs with the tile index fastest: the tiles that re-read the same
// operand rows then run on one XCD at about the same time and share its L2.
template <int TM, int TN>
__global__ void __launch_bounds__(NTHR)
wgrad_gemm_kernel(WgradDesc d0, WgradDesc d1, int tiles0, int tiles)
{
    const int nwg = gridDim.x, xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per = nwg >> 3, rem = nwg & 7;
    const int v = xcd * per + (xcd < rem ? xcd : rem) + slot;
    const int t = v % tiles, zi = v / tiles;
    constexpr bool MSPLIT = (TM / 32) * (TN / 32) > 9;  // more accumulators than one wave of a pair can hold
    if (t < tiles0) {
        if (d0.deint) wgrad_gemm_body<TM, TN, true, MSPLIT>(d0, t, zi);
        else wgrad_gemm_body<TM, TN, false, MSPLIT>(d0, t, zi);
    } else {
        if (d1.deint) wgrad_gemm_body<TM, TN, true, MSPLIT>(d1, t - tiles0, zi);
        else wgrad_gemm_body<TM, TN, false, MSPLIT>(d1, t - tiles0, zi);
    }
}

// out[g][m][col(n)] = sum_z P[z][g][m][n];  col(n) = (n % seg_w) * (N / seg_w) + n / seg_w
// (identity when seg_w == N).  Blocks [0, blocks0) reduce d0, the rest d1; eight consecutive elements per
// thread (16-byte loads of bf16 partial tiles, two 16-byte loads of fp32 ones), four chunks in flight.
// Blocks from `blocks01` on (when cj.part is set) run the second pass of the bias gradient instead.
template <bool OUT_F32>
__global__ void __launch_bounds__(256)
wgrad_reduce_kernel(WgradDesc d0, WgradDesc d1, int blocks0, int nz, ColsumJob cj, int blocks01)
{
    if ((int)blockIdx.x >= blocks01) {
        if (OUT_F32) colsum_final_body<float, 4>(cj, (int)blockIdx.x - blocks01);
        else colsum_final_body<bf16_t, 4>(cj, (int)blockIdx.x - blocks01);
        return;
    }
    const bool first = (int)blockIdx.x < blocks0;
    const WgradDesc& d = first ? d0 : d1;
    const size_t total = (size_t)d.G * d.M * d.N;  // a multiple of 8: N is a multiple of 32
    const size_t e = ((size_t)(blockIdx.x - (first ? 0 : blocks0)) * 256 + threadIdx.x) * 8;
    if (e >= total) return;
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    int z = 0;
    if (d.p_bf16) {
        const uint16_t* P = reinterpret_cast<const uint16_t*>(d.P) + e;
        for (; z + 4 <= nz; z += 4) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = ldg128(P + (size_t)(z + u) * total);
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    s[2 * w] += __uint_as_float(v[u][w] << 16);
                    s[2 * w + 1] += __uint_as_float(v[u][w] & 0xffff0000u);
                }
        }
        for (; z < nz; ++z) {
            const u32x4 v = ldg128(P + (size_t)z * total);
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                s[2 * w] += __uint_as_float(v[w] << 16);
                s[2 * w + 1] += __uint_as_float(v[w] & 0xffff0000u);
            }
        }
    } else {
        const float* P = d.P + e;
        for (; z + 4 <= nz; z += 4) {
            f32x4 v[4][2];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                v[u][0] = *reinterpret_cast<const f32x4*>(P + (size_t)(z + u) * total);
                v[u][1] = *reinterpret_cast<const f32x4*>(P + (size_t)(z + u) * total + 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int w = 0; w < 8; ++w) s[w] += v[u][w >> 2][w & 3];
        }
        for (; z < nz; ++z)
#pragma unroll
            for (int w = 0; w < 8; ++w) s[w] += P[(size_t)z * total + w];
    }
    // the eight elements share a row and (seg_w being a multiple of 8) a segment: their outputs are nseg apart
    const int nseg = d.N / d.seg_w;
    const size_t rowbase = e / d.N * d.N;
    const int n = (int)(e - rowbase);
    const size_t o = rowbase + (size_t)(n % d.seg_w) * nseg + n / d.seg_w;
    if (OUT_F32) {
        float* out = (float*)d.out + o;
        if (nseg == 1) {
            *reinterpret_cast<f32x4*>(out) = f32x4{s[0], s[1], s[2], s[3]};
            *reinterpret_cast<f32x4*>(out + 4) = f32x4{s[4], s[5], s[6], s[7]};
        } else {
#pragma unroll
            for (int w = 0; w < 8; ++w) out[(size_t)w * nseg] = s[w];
        }
    } else {
        uint16_t* out = (uint16_t*)d.out + o;
        if (nseg == 1) {
            *reinterpret_cast<u32x4*>(out) =
                u32x4{pack_bf16x2(s[0], s[1]), pack_bf16x2(s[2], s[3]), pack_bf16x2(s[4], s[5]), pack_bf16x2(s[6], s[7])};
        } else {
#pragma unroll
            for (int w = 0; w < 8; ++w) out[(size_t)w * nseg] = (uint16_t)(pack_bf16x2(s[w], 0.f) & 0xffffu);
        }
    }
}

int tiles_of(const WgradDesc& d, int tm, int tn) { return (d.M / tm) * (d.N / tn) * ((d.G + 3) / 4); }

template <int TM, int TN>
int launch_gemm(const WgradDesc& d0, const WgradDesc* d1, int nz, hipStream_t st)
{
    constexpr size_t lds = (size_t)2 * 4 * KB * (TM + lds_pad(TM) + TN + lds_pad(TN)) * 2;  // two pipeline buffers
    static_assert(lds <= kMaxLdsBytes, "LDS");
    auto kern = wgrad_gemm_kernel<TM, TN>;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess)
        return -4;
    const int t0 = tiles_of(d0, TM, TN), t1 = d1 ? tiles_of(*d1, TM, TN) : 0;
    hipLaunchKernelGGL(kern, dim3((t0 + t1) * nz), dim3(NTHR), lds, st, d0, d1 ? *d1 : d0, t0, t0 + t1);
    return hip_status(hipGetLastError());
}

int launch_gemm_tile(int tm, int tn, const WgradDesc& d0, const WgradDesc* d1, int nz, hipStream_t st)
{
#define MONARCH_WG_CASE(TM_, TN_) \
    if (tm == TM_ && tn == TN_) return launch_gemm<TM_, TN_>(d0, d1, nz, st);
    MONARCH_WG_CASE(128, 128)
    MONARCH_WG_CASE(96, 96)
    MONARCH_WG_CASE(64, 128)
    MONARCH_WG_CASE(128, 64)
    MONARCH_WG_CASE(64, 64)
    MONARCH_WG_CASE(32, 32)
#undef MONARCH_WG_CASE
    return -2;
}

}  // namespace

bool wgrad_tile_ok(int M, int N, int seg_w, int* tm, int* tn)
{
    // tile shapes instantiated above; a tile's 8-column pieces must not straddle a segment
    if (seg_w % 8 != 0) return false;
    const int cand[][2] = {{128, 128}, {96, 96}, {64, 128}, {128, 64}, {64, 64}, {32, 32}};
    for (auto& c : cand)
        if (M % c[0] == 0 && N % c[1] == 0) {
            *tm = c[0];
            *tn = c[1];
            return true;
        }
    return false;
}

int wgrad_tiles(const WgradDesc& d)
{
    int tm, tn;
    if (!wgrad_tile_ok(d.M, d.N, d.seg_w, &tm, &tn) || (d.deint && d.G != 4)) return 0;
    return tiles_of(d, tm, tn);
}

int wgrad_gemm_pair(const WgradDesc& d0, const WgradDesc& d1, int nz, hipStream_t st)
{
    int tm0, tn0, tm1, tn1;
    if (!wgrad_tile_ok(d0.M, d0.N, d0.seg_w, &tm0, &tn0) || (d0.deint && d0.G != 4)) return -2;
    if (!wgrad_tile_ok(d1.M, d1.N, d1.seg_w, &tm1, &tn1) || (d1.deint && d1.G != 4)) return -2;
    if (tm0 == tm1 && tn0 == tn1) return launch_gemm_tile(tm0, tn0, d0, &d1, nz, st);
    const int rc = launch_gemm_tile(tm0, tn0, d0, nullptr, nz, st);
    return rc ? rc : launch_gemm_tile(tm1, tn1, d1, nullptr, nz, st);
}

int wgrad_reduce_pair(const WgradDesc& d0, const WgradDesc& d1, bool out_f32, int nz, hipStream_t st, const ColsumJob* cj)
{
    if (d0.seg_w % 8 != 0 || d1.seg_w % 8 != 0 || d0.N % 8 != 0 || d1.N % 8 != 0) return -2;  // eight elements per thread
    const size_t b0 = ((size_t)d0.G * d0.M * d0.N / 8 + 255) / 256, b1 = ((size_t)d1.G * d1.M * d1.N / 8 + 255) / 256;
    ColsumJob job{};
    if (cj) job = *cj;
    const size_t b2 = cj ? (size_t)colsum_final_blocks(job) : 0;
    if (b0 + b1 + b2 > 0x7fffffffULL) return -2;
    const dim3 grid((unsigned)(b0 + b1 + b2));
    if (out_f32)
        hipLaunchKernelGGL(wgrad_reduce_kernel<true>, grid, dim3(256), 0, st, d0, d1, (int)b0, nz, job, (int)(b0 + b1));
    else
        hipLaunchKernelGGL(wgrad_reduce_kernel<false>, grid, dim3(256), 0, st, d0, d1, (int)b0, nz, job, (int)(b0 + b1));
    return hip_status(hipGetLastError());
}

}  // namespace monarch
