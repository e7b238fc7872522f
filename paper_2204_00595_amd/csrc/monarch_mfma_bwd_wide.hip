// bf16 backward for "wide block" Monarch layers (k = 4): the adjoints of steps 3, 2, P^T, 1 of
// Section 3.3 (the paper leaves them to automatic differentiation, Section 4).
//
//   prep      re-lays the weights once per call in MFMA fragment order (see prep_frag_kernel): every
//             weight operand below is then one contiguous, fully coalesced 1 KiB read per wave.
//             L is transposed with its rows picked in the order the mid permutation scatters them,
//             R is transposed with its K-slots in the order the chained accumulators of `data` hold dY1.
//   data      one workgroup per 64 batch rows, wave w <-> R block kk = w:
//               X) recompute step 1, Y1[b][kk][j] (x through a DMA-filled LDS ring, packed R fragments
//                  straight into registers), and write it to the workspace (dL needs U);
//               A) dY1[b][kk][c*Q/4 + r1] = sum_l dy[b][4*l + c] * L[c][l][4*r1 + kk]
//                  (adjoint of steps 3 + 2 + P^T in one contraction; dy is de-interleaved into
//                  LDS once per workgroup, the result stays in accumulators);
//               B) dx[b][kk*P + i] = sum_j dY1[b][kk][j] * R[kk][j][i], fed straight from the
//                  accumulators of A (converted to bf16 in registers): dY1 never goes through LDS
//                  as an operand.  dY1 is also written to the workspace for dR.
//   wgrad     dL and dR as batch-contracted GEMMs over (dy, Y1) and (dY1, x)
//             (monarch_mfma_wgrad.hip), split over the batch, then one reduction pass.
#include "monarch_internal.h"
#include "monarch_mfma_common.h"
#include "monarch_colsum.h"
#include "monarch_mfma_stage1.h"
#include "monarch_act.h"

namespace monarch {

namespace {

// ------------------------------------------------------------------------ prep ----

// The weights are re-laid once per call in MFMA *fragment order*: for every (tile, K-step) the 64
// lanes' 16-byte operand pieces are stored back to back, so that a fragment load in the data kernel
// is one contiguous, fully coalesced 1 KiB read (eight cache lines) instead of 32 or 64 lines.
// One thread builds one 16-byte piece (eight gathered elements).  Three arrays:
//   XF[kk][t][jt][lane][e]      = R[kk][32*jt + lane%32][16*t + 8*(lane/32) + e]
//       (step-1 recompute, 32x32x16: the layout stage1_block streams)
//   LF[kk][c][kt][jt][lane][e]   = L[c][32*kt + 8*(lane/16) + e][4*(16*jt + lane%16) + kk]
//       (dY1 stage, 16x16x32: L transposed, rows picked as the mid permutation scatters them)
//   RF[kk][ig][u][it][lane][e]   = R[kk][32*u + 16*(e/4) + 4*(lane/16) + e%4][16*(ig*IG + it) + lane%16]
//       (dx stage, 16x16x32: R transposed, K-slots in the order the chained accumulators hold dY1)
__global__ void __launch_bounds__(256)
prep_frag_kernel(const uint16_t* __restrict__ L, const uint16_t* __restrict__ R, uint16_t* __restrict__ XF,
                 uint16_t* __restrict__ LF, uint16_t* __restrict__ RF, int P, int Q, int S, int JG, int IG,
                 ColsumJob cj, int nprep)
{
    // workgroups past the re-layout run the first pass of the bias gradient (column sums of dy)
    if ((int)blockIdx.x >= nprep) {
        colsum_partial_body<bf16_t, 4>(cj, (int)blockIdx.x - nprep);
        return;
    }
    const int nR = 4 * Q * P / 8, nL = 4 * S * Q / 8;  // pieces per array
    int pc = blockIdx.x * 256 + threadIdx.x;
    uint16_t v[8];
    uint16_t* dst;
    if (pc < nR) {
        const int lane = pc & 63;
        int rest = pc >> 6;
        const int QT = Q / 32, T = P / 16;
        const int jt = rest % QT; rest /= QT;
        const int t = rest % T, kk = rest / T;
        const uint16_t* src = R + ((size_t)kk * Q + 32 * jt + (lane & 31)) * P + 16 * t + 8 * (lane >> 5);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[e];
        dst = XF + (size_t)pc * 8;
    } else if (pc < nR + nL) {
        pc -= nR;
        const int lane = pc & 63;
        int rest = pc >> 6;
        const int JT = Q / 4 / 16;
        const int jt = rest % JT; rest /= JT;
        const int KT = S / 32;
        const int kt = rest % KT; rest /= KT;
        const int c = rest & 3, kk = rest >> 2;
        const uint16_t* src = L + ((size_t)c * S + 32 * kt + 8 * (lane >> 4)) * Q + 4 * (16 * jt + (lane & 15)) + kk;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[(size_t)e * Q];
        dst = LF + (size_t)pc * 8;
    } else if (pc < 2 * nR + nL) {
        pc -= nR + nL;
        const int lane = pc & 63;
        int rest = pc >> 6;
        const int it = rest % IG; rest /= IG;
        const int U = Q / 32;
        const int u = rest % U; rest /= U;
        const int nig = P / 16 / IG;
        const int ig = rest % nig, kk = rest / nig;
        const uint16_t* src = R + ((size_t)kk * Q + 32 * u + 4 * (lane >> 4)) * P + 16 * (ig * IG + it) + (lane & 15);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[(size_t)(16 * (e >> 2) + (e & 3)) * P];
        dst = RF + (size_t)pc * 8;
    } else {
        return;
    }
    u32x4 o;
#pragma unroll
    for (int w = 0; w < 4; ++w) o[w] = (uint32_t)v[2 * w] | ((uint32_t)v[2 * w + 1] << 16);
    *reinterpret_cast<u32x4*>(dst) = o;
}

// ------------------------------------------------------------------------ data ----

template <int P_, int Q_, int S_, int JG_, int LC_, int IG_>
struct BwdWide {
    static constexpr int K = 4, P = P_, Q = Q_, S = S_, JG = JG_, LC = LC_, IG = IG_;
    static constexpr int BM = 64, NB = 2;   // stage X uses 32 x 32 tiles (2 row tiles)
    static constexpr int NBT = 4;           // stages A, B use 16 x 16 tiles (4 row tiles)
    static constexpr int QK = Q / K, QT = Q / 32, KQ = K * Q;
    static constexpr int N_IN = K * P, N_OUT = K * S;
    static constexpr int JT = QK / 16;      // 16-wide j tiles per (kk, c)
    static constexpr int Y1_STRIDE = KQ + 8;
    static constexpr int DW_STRIDE = LC + 8;
    static constexpr int DX_COLS = IG * 16;          // dx columns staged per wave at a time
    static constexpr int DX_STRIDE = DX_COLS + 8;
    static constexpr size_t LDS_Y1 = (size_t)BM * Y1_STRIDE * 2;
    static constexpr size_t LDS_DW = (size_t)K * BM * DW_STRIDE * 2;
    static constexpr size_t LDS_DX = (size_t)4 * BM * DX_STRIDE * 2;
    using S1 = Stage1<P_, Q_>;               // step-1 recompute (x through an LDS ring, packed R fragments)
    static constexpr size_t max2(size_t a, size_t b) { return a > b ? a : b; }
    static constexpr size_t LDS_BYTES = max2(max2(LDS_Y1, LDS_DW), max2(LDS_DX, S1::LDS_X));
    static_assert(P % 64 == 0 && Q % 32 == 0 && S % 32 == 0 && QK % 16 == 0, "tile shapes");
    static_assert(QT % JG == 0 && S % LC == 0 && LC % 32 == 0 && (P / 16) % IG == 0, "loop splits");
    static_assert(DX_COLS % 8 == 0 && (64 % (DX_COLS / 8) == 0), "dx staging copy-out");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

// cooperative copy of a [64][COLS] bf16 LDS tile (row stride `stride`) to global rows b0.. (row pitch ld);
// eight LDS reads are in flight per thread before the first store.  NT: streaming (non-temporal) stores.
template <int COLS, int NTHREADS, bool NT>
__device__ __forceinline__ void copy_out_tile(const uint16_t* src, int stride, uint16_t* dst, int64_t ld,
                                              int64_t b0, int64_t B, int tid)
{
    constexpr int PER_ROW = COLS / 8, TASKS = 64 * PER_ROW, PER = (TASKS + NTHREADS - 1) / NTHREADS;
    // the rounds are not unrolled: unrolled, the compiler precomputes every round's addresses and, next
    // to the accumulators that are live around the copies, spills them
#pragma unroll 1
    for (int i0 = 0; i0 < PER; i0 += 8) {
        u32x4 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t = tid + (i0 + i) * NTHREADS;
            if (i0 + i < PER && t < TASKS) v[i] = lds128(src + (size_t)(t / PER_ROW) * stride + 8 * (t % PER_ROW));
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t = tid + (i0 + i) * NTHREADS;
            const int r = t / PER_ROW, u = t % PER_ROW;
            if (i0 + i < PER && t < TASKS && b0 + r < B) {
                uint16_t* p = dst + (b0 + r) * ld + 8 * u;
                if (NT) stg128_nt(p, v[i]);
                else *reinterpret_cast<u32x4*>(p) = v[i];
            }
        }
    }
}

// The wave-private dx tile ([64][COLS] bf16 in LDS) goes out multiplied elementwise by gelu'(x_pre): the layer's
// input was gelu(x_pre) and the caller wants the gradient with respect to x_pre.  Lane task i is row
// lane / (COLS/8) + (512/COLS) * i, 16-byte piece lane % (COLS/8); `pre` holds the x_pre pieces of the same tasks
// (fetched by load_pre_tile before the MFMA loop, so that their latency is hidden).
template <int COLS>
__device__ __forceinline__ void load_pre_tile(const uint16_t* pre, int64_t ld, int64_t b0, int64_t B, int lane,
                                              u32x4 (&hp)[COLS / 8])
{
    constexpr int PER_ROW = COLS / 8;
    static_assert(64 % PER_ROW == 0, "whole rows per round");
#pragma unroll
    for (int i = 0; i < PER_ROW; ++i) {
        const int t = lane + i * 64;
        int64_t row = b0 + t / PER_ROW;
        row = row < B ? row : B - 1;  // rows past the end are read from a valid row and never stored
        hp[i] = ldg128_nt(pre + row * ld + 8 * (t % PER_ROW));
    }
}

template <int COLS>
__device__ __forceinline__ void copy_out_tile_gelu(const uint16_t* src, int stride, uint16_t* dst, int64_t ld,
                                                   int64_t b0, int64_t B, int lane, const u32x4 (&hp)[COLS / 8])
{
    constexpr int PER_ROW = COLS / 8;
#pragma unroll
    for (int i = 0; i < PER_ROW; ++i) {
        const int t = lane + i * 64;
        const int r = t / PER_ROW, u = t % PER_ROW;
        const u32x4 v = lds128(src + (size_t)r * stride + 8 * u);
        u32x4 o;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float g0 = __uint_as_float(v[w] << 16), g1 = __uint_as_float(v[w] & 0xffff0000u);
            const float h0 = __uint_as_float(hp[i][w] << 16), h1 = __uint_as_float(hp[i][w] & 0xffff0000u);
            o[w] = pack_bf16x2(g0 * gelu_grad_f(h0), g1 * gelu_grad_f(h1));
        }
        if (b0 + r < B) stg128_nt(dst + (b0 + r) * ld + 8 * u, o);
    }
}

// orders the LDS traffic of one wave (what its lanes wrote is visible to its later reads)
__device__ __forceinline__ void wave_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// MODE 0: everything.  MODE 1: the transposed multiply y = x M on its own (dy is then the input x of
// that product, dx its output): the recompute of step 1 and the workspace copies of both intermediates
// are left out.  MODE 2: the forward saved the vector between the factors, so step 1 is not recomputed;
// dY1 still goes to the workspace for the weight-gradient GEMM.
// ACT: dx leaves multiplied by gelu'(x_pre) (the layer's input was x = gelu(x_pre)).
template <typename C, int MODE, bool ACT>
__global__ void __launch_bounds__(256)
bwd_wide_data_kernel(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ x,
                     const uint16_t* __restrict__ XF, const uint16_t* __restrict__ LF,
                     const uint16_t* __restrict__ RF, uint16_t* __restrict__ dx,
                     uint16_t* __restrict__ Y1ws, uint16_t* __restrict__ dY1ws, const uint16_t* __restrict__ x_pre,
                     int64_t B)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;
    const int kk = wave;

    // dy is consumed in chunks of LC features l; a chunk (64 rows x 4*LC columns) is fetched into
    // registers well before it is de-interleaved into LDS, so that its HBM latency is hidden
    constexpr int RUNS = C::LC / 8;                 // 64-byte runs per row and chunk
    constexpr int DYT = 64 * RUNS / 256;            // runs per thread
    static_assert(64 * RUNS % 256 == 0, "dy chunk split");
    u32x4 raw[DYT][4];
    auto load_dy = [&](int l0) {
#pragma unroll
        for (int i = 0; i < DYT; ++i) {
            const int t = tid + i * 256;
            const int r = t / RUNS, u = t - r * RUNS;
            int64_t row = b0 + r;
            row = row < B ? row : B - 1;
            const uint16_t* p = dy + row * C::N_OUT + (size_t)(l0 + 8 * u) * 4;
#pragma unroll
            for (int w = 0; w < 4; ++w) raw[i][w] = ldg128(p + 8 * w);  // cached: the weight-gradient GEMM re-reads dy
        }
    };

    // ------------------------------------------------- X: recompute step 1 -> workspace ----
    if constexpr (MODE != 0) {
        load_dy(0);
    } else {
        const int ln = lane & 31, g = lane >> 5;
        f32x16 acc[C::QT * C::NB];
        stage1_block<typename C::S1>(x, XF, b0, B, kk, lane, lds + (size_t)wave * C::S1::XR * 4096, acc);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();  // every wave is done with its x ring: the space becomes the Y1 tile
        // lane holds D^T[j][b] for b = nb*32 + ln and j = jt*32 + 8*(i/4) + 4*g + i%4
#pragma unroll
        for (int jt = 0; jt < C::QT; ++jt)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x16& a = acc[jt * C::NB + nb];
                    u32x2 v = {pack_bf16x2(a[4 * i4 + 0], a[4 * i4 + 1]), pack_bf16x2(a[4 * i4 + 2], a[4 * i4 + 3])};
                    const int j = jt * 32 + 8 * i4 + 4 * g;
                    *reinterpret_cast<u32x2*>(lds + (size_t)(nb * 32 + ln) * C::Y1_STRIDE + kk * C::Q + j) = v;
                }
        load_dy(0);  // in flight during the copy-out below
        __syncthreads();
        copy_out_tile<C::KQ, 256, false>(lds, C::Y1_STRIDE, Y1ws, C::KQ, b0, B, tid);
        __syncthreads();
    }

    // 16 x 16 tile coordinates for stages A and B
    const int l16 = lane & 15, h = lane >> 4;

    // ------------------------------------------------- A: dY1 (accumulators) ----
    // accA[(c*JT + jt)*NBT + bt][e] = dY1[b = bt*16 + l16][kk][j = c*QK + jt*16 + 4*h + e]
    f32x4 accA[C::K * C::JT * C::NBT];
#pragma unroll
    for (int t = 0; t < C::K * C::JT * C::NBT; ++t) accA[t] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int l0 = 0; l0 < C::S; l0 += C::LC) {
        // A operand: fragment (c, kt, jt) of LF (rows kk*QK + jt*16 + l16 of L^T), streamed through a
        // ring of NSA K-steps over the flattened (c, t) loop; the first loads are issued before the
        // de-interleave below so that they overlap it.
        constexpr int T = C::LC / 32, NSA = 4, NSTEP = C::K * T;
        const uint16_t* Lk = LF + (((size_t)kk * 4 * (C::S / 32) + l0 / 32) * C::JT * 64 + lane) * 8;
        u32x4 af[NSA][C::JT];
        auto issue = [&](int n, int slot) {
            const int c = n / T, t = n % T;
#pragma unroll
            for (int jt = 0; jt < C::JT; ++jt)
                af[slot][jt] = ldg128(Lk + ((size_t)(c * (C::S / 32) + t) * C::JT + jt) * 512);
        };
#pragma unroll
        for (int d = 0; d < NSA - 1; ++d)
            if (d < NSTEP) issue(d, d);
        __builtin_amdgcn_sched_barrier(0);
        // de-interleave the chunk (loaded earlier, see load_dy) into LDS dWs[c][b][l - l0]
#pragma unroll
        for (int i = 0; i < DYT; ++i) {
            const int t = tid + i * 256;
            const int r = t / RUNS, u = t - r * RUNS;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                u32x4 v;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t lo = raw[i][w][c >> 1], hi = raw[i][w][2 + (c >> 1)];
                    v[w] = (c & 1) ? pick_hi16(lo, hi) : pick_lo16(lo, hi);
                }
                *reinterpret_cast<u32x4*>(lds + ((size_t)c * 64 + r) * C::DW_STRIDE + 8 * u) = v;
            }
        }
        __syncthreads();
        if (l0 + C::LC < C::S) load_dy(l0 + C::LC);  // the next chunk is in flight during the MFMA loop
#pragma unroll
        for (int n = 0; n < NSTEP; ++n) {
            const int c = n / T, t = n % T;
            __builtin_amdgcn_sched_barrier(0);
            if (n + NSA - 1 < NSTEP) issue(n + NSA - 1, (n + NSA - 1) % NSA);
            __builtin_amdgcn_sched_barrier(0);
            // B operand: dWs[c][bt*16 + l16][l]
            const uint16_t* Wc = lds + ((size_t)c * 64 + l16) * C::DW_STRIDE + 8 * h;
            bf16x8 bfr[C::NBT];
#pragma unroll
            for (int bt = 0; bt < C::NBT; ++bt)
                bfr[bt] = as_bf16x8(lds128(Wc + (size_t)bt * 16 * C::DW_STRIDE + t * 32));
#pragma unroll
            for (int jt = 0; jt < C::JT; ++jt)
#pragma unroll
                for (int bt = 0; bt < C::NBT; ++bt)
                    accA[(c * C::JT + jt) * C::NBT + bt] =
                        mfma16(as_bf16x8(af[n % NSA][jt]), bfr[bt], accA[(c * C::JT + jt) * C::NBT + bt]);
        }
        __syncthreads();
    }
    // bf16 fragments of dY1: dfr[J][bt] holds j = J*16 + 4*h + 0..3 (J = c*JT + jt) for row bt*16 + l16
    u32x2 dfr[C::K * C::JT][C::NBT];
#pragma unroll
    for (int J = 0; J < C::K * C::JT; ++J)
#pragma unroll
        for (int bt = 0; bt < C::NBT; ++bt) {
            const f32x4& a = accA[J * C::NBT + bt];
            dfr[J][bt] = u32x2{pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3])};
        }
    // dY1 -> workspace through LDS (natural layout [b][kk*Q + j])
    if constexpr (MODE != 1) {
#pragma unroll
        for (int J = 0; J < C::K * C::JT; ++J)
#pragma unroll
            for (int bt = 0; bt < C::NBT; ++bt)
                *reinterpret_cast<u32x2*>(lds + (size_t)(bt * 16 + l16) * C::Y1_STRIDE + kk * C::Q + J * 16 + 4 * h) = dfr[J][bt];
        __syncthreads();
        copy_out_tile<C::KQ, 256, false>(lds, C::Y1_STRIDE, dY1ws, C::KQ, b0, B, tid);
        __syncthreads();
    }

    // ------------------------------------------------- B: dx from the chained fragments ----
    // K-step u covers j in [32u, 32u+32): lane slots 0..3 <- tile 2u, slots 4..7 <- tile 2u+1;
    // the RF fragments are laid out in exactly that order.
    uint16_t* stage = lds + (size_t)wave * 64 * C::DX_STRIDE;
    constexpr int U = C::Q / 32;
    const uint16_t* Rt = RF + ((size_t)kk * (C::P / 16 / C::IG) * U * C::IG * 64 + lane) * 8;
    // The fragments of all (ig, u) steps are contiguous in RF: step n = ig*U + u.  They run through a
    // ring of NSB steps that continues across the ig loop (U % NSB == 0 keeps the slot numbers static).
    constexpr int NIG = (C::P / 16) / C::IG;
    constexpr int NSB = (U % 4 == 0) ? 4 : ((U % 3 == 0) ? 3 : 2);
    static_assert(U % NSB == 0, "ring");
    u32x4 af[NSB][C::IG];
    auto issue = [&](int n, int slot) {
#pragma unroll
        for (int it = 0; it < C::IG; ++it) af[slot][it] = ldg128(Rt + ((size_t)n * C::IG + it) * 512);
    };
#pragma unroll
    for (int d = 0; d < NSB - 1; ++d) issue(d, d);
    for (int ig = 0; ig < NIG; ++ig) {
        f32x4 acc[C::IG * C::NBT];
#pragma unroll
        for (int t = 0; t < C::IG * C::NBT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        u32x4 hp[C::DX_COLS / 8];
        if constexpr (ACT) load_pre_tile<C::DX_COLS>(x_pre + kk * C::P + ig * C::DX_COLS, C::N_IN, b0, B, lane, hp);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int n = ig * U + u;
            __builtin_amdgcn_sched_barrier(0);
            if (n + NSB - 1 < NIG * U) issue(n + NSB - 1, (u + NSB - 1) % NSB);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int bt = 0; bt < C::NBT; ++bt) {
                const u32x4 bv = {dfr[2 * u][bt][0], dfr[2 * u][bt][1], dfr[2 * u + 1][bt][0], dfr[2 * u + 1][bt][1]};
                const bf16x8 bfr = as_bf16x8(bv);
#pragma unroll
                for (int it = 0; it < C::IG; ++it)
                    acc[it * C::NBT + bt] = mfma16(as_bf16x8(af[u % NSB][it]), bfr, acc[it * C::NBT + bt]);
            }
        }
        // D^T[i][b]: lane holds i = it*16 + 4*h + 0..3 for row b = bt*16 + l16
#pragma unroll
        for (int it = 0; it < C::IG; ++it)
#pragma unroll
            for (int bt = 0; bt < C::NBT; ++bt) {
                const f32x4& a = acc[it * C::NBT + bt];
                *reinterpret_cast<u32x2*>(stage + (size_t)(bt * 16 + l16) * C::DX_STRIDE + it * 16 + 4 * h) =
                    u32x2{pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3])};
            }
        // the staging tile is private to the wave: no workgroup barrier
        wave_fence();
        if constexpr (ACT)
            copy_out_tile_gelu<C::DX_COLS>(stage, C::DX_STRIDE, dx + kk * C::P + ig * C::DX_COLS, C::N_IN, b0, B, lane, hp);
        else
            copy_out_tile<C::DX_COLS, 64, true>(stage, C::DX_STRIDE, dx + kk * C::P + ig * C::DX_COLS, C::N_IN, b0, B, lane);
        wave_fence();
    }
}

template <typename C>
int launch_data(const Problem& pb, const void* dy, const void* x, const uint16_t* XF, const uint16_t* LF,
                const uint16_t* RF, void* dx, uint16_t* Y1ws, uint16_t* dY1ws, hipStream_t st)
{
    // no workspace for dY1: dx only; dY1 but no Y1 workspace: the forward saved that vector
    // (the nonlinearity's factor is applied here only by the recomputing backward)
    auto kern = !dY1ws ? bwd_wide_data_kernel<C, 1, false>
                       : (Y1ws ? (pb.x_pre ? bwd_wide_data_kernel<C, 0, true> : bwd_wide_data_kernel<C, 0, false>)
                               : (pb.x_pre ? bwd_wide_data_kernel<C, 2, true> : bwd_wide_data_kernel<C, 2, false>));
    if (pb.x_pre && !dY1ws) return -2;
    if (allow_dynamic_lds((const void*)kern, C::LDS_BYTES) != hipSuccess)
        return -4;
    const int64_t grid = (pb.B + C::BM - 1) / C::BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), C::LDS_BYTES, st, (const uint16_t*)dy,
                       (const uint16_t*)x, XF, LF, RF, (uint16_t*)dx, Y1ws, dY1ws, (const uint16_t*)pb.x_pre, pb.B);
    return hip_status(hipGetLastError());
}

struct Entry {
    int p, q, s, jg, ig;  // jg, ig: the data kernel's loop splits, which fix the fragment order of the weights
    int (*fn)(const Problem&, const void*, const void*, const uint16_t*, const uint16_t*, const uint16_t*, void*,
              uint16_t*, uint16_t*, hipStream_t);
};

//                                 P     Q     S   JG   LC  IG
const Entry kTable[] = {
    {192, 192, 192, 6, 4, launch_data<BwdWide<192, 192, 192, 6, 192, 4>>},
    {192, 192, 768, 6, 4, launch_data<BwdWide<192, 192, 768, 6, 192, 4>>},
    {256, 256, 1024, 4, 4, launch_data<BwdWide<256, 256, 1024, 4, 128, 4>>},
    {1024, 256, 256, 4, 4, launch_data<BwdWide<1024, 256, 256, 4, 128, 4>>},
    {768, 192, 192, 6, 4, launch_data<BwdWide<768, 192, 192, 6, 192, 4>>},
    {256, 256, 256, 4, 4, launch_data<BwdWide<256, 256, 256, 4, 128, 4>>},
    {192, 192, 576, 6, 4, launch_data<BwdWide<192, 192, 576, 6, 192, 4>>},
    {256, 256, 768, 4, 4, launch_data<BwdWide<256, 256, 768, 4, 128, 4>>},
    {128, 128, 128, 4, 4, launch_data<BwdWide<128, 128, 128, 4, 128, 4>>},
    {128, 128, 512, 4, 4, launch_data<BwdWide<128, 128, 512, 4, 128, 4>>},
    {512, 128, 128, 4, 4, launch_data<BwdWide<512, 128, 128, 4, 128, 4>>},
    {64, 64, 64, 2, 4, launch_data<BwdWide<64, 64, 64, 2, 64, 4>>},
    {64, 64, 128, 2, 4, launch_data<BwdWide<64, 64, 128, 2, 64, 4>>},
    {128, 64, 64, 2, 4, launch_data<BwdWide<128, 64, 64, 2, 64, 4>>},
};

const Entry* find(const Problem& pb)
{
    if (pb.dtype != 1 || pb.k != 4 || pb.perm_b()) return nullptr;
    for (const Entry& e : kTable)
        if (e.p == pb.p && e.q == pb.q && e.s == pb.s) return &e;
    return nullptr;
}

// The two weight-gradient GEMMs share one split of the batch into nz chunks: about one
// workgroup per CU in total, chunks of at least 256 rows (multiples of the 32-row pipeline
// step) so that the fp32 partial tiles stay small next to the operands.
struct Plan {
    size_t off_y1, off_dy1, off_xf, off_lf, off_rf, off_partL, off_partR, total;
    int nz, rows_per_chunk;
    bool ok;
};

void fill_descs(const Problem& pb, WgradDesc& dl, WgradDesc& dr)
{
    // dL[c][l][4*r1 + kk] = sum_b dy[b][4*l + c] * Y1[b][kk][c*Q/4 + r1]
    dl = WgradDesc{};
    dl.lda = pb.n_out(); dl.a_g = 1; dl.deint = 1;
    dl.ldb = pb.kq(); dl.b_g = pb.q / 4; dl.b_seg = pb.q; dl.seg_w = pb.q / 4;
    dl.M = pb.s; dl.N = pb.q; dl.G = 4; dl.rows = pb.B;
    // dR[kk][j][i] = sum_b dY1[b][kk][j] * x[b][kk*P + i]
    dr = WgradDesc{};
    dr.lda = pb.kq(); dr.a_g = pb.q; dr.deint = 0;
    dr.ldb = pb.n_in; dr.b_g = pb.p; dr.b_seg = 0; dr.seg_w = pb.p;
    dr.M = pb.q; dr.N = pb.p; dr.G = 4; dr.rows = pb.B;
}

Plan make_plan(const Problem& pb)
{
    Plan pl{};
    WgradDesc dl, dr;
    fill_descs(pb, dl, dr);
    const int tiles = wgrad_tiles(dl) + wgrad_tiles(dr);
    pl.ok = wgrad_tiles(dl) > 0 && wgrad_tiles(dr) > 0;
    if (!pl.ok) return pl;
    int64_t z = 256 / tiles;  // one workgroup (eight waves) per CU: its two LDS buffers leave room for one only
    const int64_t maxz = (pb.B + 255) / 256;
    if (z > maxz) z = maxz;
    if (z < 1) z = 1;
    const int64_t rpc = ((pb.B + z - 1) / z + 63) / 64 * 64;  // whole pipeline rounds (two 32-row steps)
    pl.rows_per_chunk = (int)(rpc > 0 ? rpc : 32);
    pl.nz = (int)((pb.B + pl.rows_per_chunk - 1) / pl.rows_per_chunk);
    if (pl.nz < 1) pl.nz = 1;
    size_t off = 0;
    const size_t act = align_up((size_t)(pb.B > 0 ? pb.B : 1) * pb.kq() * 2, 256);
    pl.off_y1 = off;  off += act;
    pl.off_dy1 = off; off += act;
    pl.off_xf = off; off += align_up(pb.n_R() * 2, 256);
    pl.off_lf = off; off += align_up(pb.n_L() * 2, 256);
    pl.off_rf = off; off += align_up(pb.n_R() * 2, 256);
    pl.off_partL = off; off += align_up((size_t)pl.nz * pb.n_L() * 4, 256);
    pl.off_partR = off; off += align_up((size_t)pl.nz * pb.n_R() * 4, 256);
    pl.total = off;
    return pl;
}

}  // namespace

bool bwd_wide_supported(const Problem& pb) { return find(pb) != nullptr && make_plan(pb).ok; }
bool saved_supported(const Problem& pb) { return bwd_wide_supported(pb) && fwd_wide_supported(pb); }

// Transposed multiply through the same data kernel (the weights in fragment order, then the dx stages).
size_t fwd_t_wide_workspace(const Problem& pb) { return 2 * align_up(pb.n_R() * 2, 256) + align_up(pb.n_L() * 2, 256); }

int fwd_t_wide(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    const Entry* e = find(pb);
    if (!e) return -2;
    char* w = (char*)ws;
    uint16_t* XF = (uint16_t*)w;
    uint16_t* LF = (uint16_t*)(w + align_up(pb.n_R() * 2, 256));
    uint16_t* RF = (uint16_t*)(w + align_up(pb.n_R() * 2, 256) + align_up(pb.n_L() * 2, 256));
    const size_t pieces = (2 * pb.n_R() + pb.n_L()) / 8;
    const int nprep = (int)((pieces + 255) / 256);
    hipLaunchKernelGGL(prep_frag_kernel, dim3((unsigned)nprep), dim3(256), 0, st, (const uint16_t*)L, (const uint16_t*)R,
                       XF, LF, RF, pb.p, pb.q, pb.s, e->jg, e->ig, ColsumJob{}, nprep);
    if (hipGetLastError() != hipSuccess) return -4;
    return e->fn(pb, x, nullptr, XF, LF, RF, y, nullptr, nullptr, st);
}

size_t bwd_wide_workspace(const Problem& pb) { return make_plan(pb).total; }

int bwd_wide(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx,
             void* dR, void* dL, void* ws, hipStream_t st)
{
    const Entry* e = find(pb);
    const Plan pl = make_plan(pb);
    if (!e || !pl.ok) return -2;
    char* w = (char*)ws;
    uint16_t* Y1ws = (uint16_t*)(w + pl.off_y1);
    uint16_t* dY1ws = (uint16_t*)(w + pl.off_dy1);
    uint16_t* XF = (uint16_t*)(w + pl.off_xf);
    uint16_t* LF = (uint16_t*)(w + pl.off_lf);
    uint16_t* RF = (uint16_t*)(w + pl.off_rf);
    const bool f32out = pb.wgrad_f32();
    if (pb.B == 0) {
        int rc = f32out ? launch_fill_zero_f32((float*)dR, pb.n_R(), st) : launch_fill_zero_u16((uint16_t*)dR, pb.n_R(), st);
        if (rc) return rc;
        return f32out ? launch_fill_zero_f32((float*)dL, pb.n_L(), st) : launch_fill_zero_u16((uint16_t*)dL, pb.n_L(), st);
    }
    const size_t pieces = (2 * pb.n_R() + pb.n_L()) / 8;
    const int nprep = (int)((pieces + 255) / 256);
    ColsumJob cj{};
    const bool want_db = pb.dbias != nullptr;
    if (want_db) cj = make_colsum_job(pb, dy, pb.dbias, pb.colsum_ws);
    hipLaunchKernelGGL(prep_frag_kernel, dim3((unsigned)(nprep + (want_db ? colsum_partial_blocks(cj) : 0))), dim3(256), 0,
                       st, (const uint16_t*)L, (const uint16_t*)R, XF, LF, RF, pb.p, pb.q, pb.s, e->jg, e->ig, cj, nprep);
    if (hipGetLastError() != hipSuccess) return -4;
    // Step 1 (Y1, for dL) is recomputed either by the data kernel itself or, for the shapes that have it, by a
    // GEMM of its own with four times the rows per workgroup (monarch_mfma_y1.hip); not at all when the forward saved it.
    const bool y1_apart = !pb.saved && y1_gemm_supported(pb);
    int rc = 0;
    if (y1_apart) {
        rc = y1_gemm(pb, x, XF, Y1ws, st);
        if (rc) return rc;
    }
    rc = e->fn(pb, dy, x, XF, LF, RF, dx, (pb.saved || y1_apart) ? nullptr : Y1ws, dY1ws, st);
    if (rc) return rc;

    WgradDesc dl, dr;
    fill_descs(pb, dl, dr);
    dl.A = (const uint16_t*)dy; dl.Bm = Y1ws; dl.P = (float*)(w + pl.off_partL); dl.out = dL;
    if (pb.saved) {
        // the saved vector is in stage-2 order: group c owns the Q contiguous columns c*Q .. of every row
        dl.Bm = (const uint16_t*)pb.saved;
        dl.b_g = pb.q; dl.b_seg = 0; dl.seg_w = pb.q;
    }
    dr.A = dY1ws; dr.Bm = (const uint16_t*)x; dr.P = (float*)(w + pl.off_partR); dr.out = dR;
    dl.rows_per_chunk = dr.rows_per_chunk = pl.rows_per_chunk;
    dl.p_bf16 = dr.p_bf16 = f32out ? 0 : 1;  // bf16 gradients: bf16 partial tiles
    rc = wgrad_gemm_pair(dl, dr, pl.nz, st);
    if (rc) return rc;
    return wgrad_reduce_pair(dl, dr, f32out, pl.nz, st, want_db ? &cj : nullptr);
}

}  // namespace monarch
