// Fused bf16 forward for "wide block" Monarch layers (k = 4 blocks, block sizes that are
// multiples of 32): both block-diagonal stages of Section 3.3 on v_mfma_f32_32x32x16_bf16,
// the mid permutation P^T folded into operand addressing, the intermediate in LDS only.
//
// One workgroup (4 waves) owns BM = 64 batch rows.
//
// Stage 1  (step 1 of Section 3.3): wave w computes block kk = w,
//     Y1[b][kk][j] = sum_i R[kk][j][i] x[b][kk*P + i],
// as D^T = R . X^T so that each lane ends up with 4 consecutive j for one row b and can
// write them to LDS as one 8-byte store.  R and x fragments go global -> registers directly
// (every byte is needed by exactly one wave, so LDS staging would only add traffic).
// LDS holds Y1s[b][kk*Q + j] in bf16, i.e. the natural (k, q) grid, not yet permuted.
//
// Stage 2  (step 2): block c contracts over r = 0..Q-1 with
//     U[b][c*Q + r] = Y1[b][r % 4][c*Q/4 + r/4]      (P^T of Definition 3.1 on the (4, Q) grid).
// The contraction order is free, so it runs over (kk, r1) with r = 4*r1 + kk: the A operand is
// then 8 consecutive bf16 of Y1s (one ds_read_b128), and the B operand is every 4th element of
// a 64-byte run of an L row, picked out of four global_load_dwordx4 with v_perm_b32.  No data
// is ever moved to apply the permutation.
// Waves split the output features l; each wave keeps all four c for its l-tile so that
// step 3, y[b][4*l + c], becomes one packed 8-byte store per (b, l): 256 contiguous bytes
// per 32 lanes.
#include "monarch_internal.h"
#include "monarch_mfma_common.h"

namespace monarch {

namespace {

template <int P_, int Q_, int S_, int BM_, int JG_>
struct FwdWide {
    static constexpr int K = 4, P = P_, Q = Q_, S = S_, BM = BM_, JG = JG_;
    static constexpr int NB = BM / 32;       // 32-row tiles per workgroup
    static constexpr int QK = Q / K;         // columns of each R block that feed one L block
    static constexpr int QT = Q / 32;        // j-tiles per R block
    static constexpr int ST = S / 32;        // l-tiles per L block
    static constexpr int KQ = K * Q;
    static constexpr int N_IN = K * P;
    static constexpr int N_OUT = K * S;
    static constexpr int LDS_STRIDE = KQ + 8;  // bf16 elements; +16 bytes keeps ds_read_b128 conflict-free
    static constexpr size_t LDS_BYTES = (size_t)BM * LDS_STRIDE * 2;
    static constexpr int ROUNDS = ST / 4;    // l-tiles handled whole, one per wave per round
    static constexpr int REM = ST % 4;       // left-over l-tiles, split by 32-row tile across waves
    static_assert(BM % 32 == 0 && P % 16 == 0 && Q % 32 == 0 && S % 32 == 0, "tile shapes");
    static_assert(QK % 16 == 0, "stage-2 K-chunks cover 16 columns of every R block");
    static_assert(QT % JG == 0, "j-tile groups");
    static_assert(REM == 0 || (REM == 2 && NB == 2), "left-over l-tiles are split two waves per tile");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

template <int N>
__device__ __forceinline__ void zero_acc(f32x16 (&a)[N])
{
#pragma unroll
    for (int n = 0; n < N; ++n)
#pragma unroll
        for (int i = 0; i < 16; ++i) a[n][i] = 0.f;
}

// Stage 2 for l-tile `lt` and the NBL 32-row tiles starting at nb0.
template <typename C, int NBL>
__device__ __forceinline__ void stage2_tile(const uint16_t* __restrict__ L, const uint16_t* y1s,
                                            uint16_t* __restrict__ y, int64_t b0, int64_t B, int lt,
                                            int nb0, int ln, int g)
{
    constexpr int K = 4;
    constexpr int NV = C::QK / 16;  // 64-byte runs of an L row per 16 columns of every R block
    constexpr int NCH = K * NV;     // runs per l-tile
    f32x16 acc[K * NBL];
    zero_acc(acc);

    // L[c][l][r]: this lane owns row l = lt*32 + ln and, in run v, elements r in [(16v + 8g)*4, +32)
    const uint16_t* Lbase = L + (size_t)(lt * 32 + ln) * C::Q + 32 * g;
    const uint16_t* abase = y1s + (size_t)(nb0 * 32 + ln) * C::LDS_STRIDE + 8 * g;

    // Ring of PF+1 register buffers, one 64-byte run each: run ch+PF is requested before the
    // MFMAs of run ch are issued.  The scheduling barriers keep the compiler from hoisting every
    // load of the (fully unrolled) loop to the top, which would not fit the register file.
    constexpr int PF = 2;
    u32x4 raw[PF + 1][4];
    auto load_run = [&](int ch, u32x4 (&dst)[4]) {
        const uint16_t* p = Lbase + (size_t)(ch / NV) * C::S * C::Q + (ch % NV) * 64;
#pragma unroll
        for (int d = 0; d < 4; ++d) dst[d] = ldg128(p + 8 * d);
    };
#pragma unroll
    for (int ch = 0; ch < PF && ch < NCH; ++ch) load_run(ch, raw[ch]);
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
        __builtin_amdgcn_sched_barrier(0);
        if (ch + PF < NCH) load_run(ch + PF, raw[(ch + PF) % (PF + 1)]);
        const int c = ch / NV, v = ch % NV;
        const u32x4(&rw)[4] = raw[ch % (PF + 1)];
#pragma unroll
        for (int kk = 0; kk < K; ++kk) {
            // elements kk, kk+4, ..., kk+28 of the run
            u32x4 bf;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t lo = rw[w][kk >> 1], hi = rw[w][2 + (kk >> 1)];
                bf[w] = (kk & 1) ? pick_hi16(lo, hi) : pick_lo16(lo, hi);
            }
            const bf16x8 bfrag = as_bf16x8(bf);
#pragma unroll
            for (int nb = 0; nb < NBL; ++nb) {
                const bf16x8 afrag =
                    as_bf16x8(lds128(abase + (size_t)nb * 32 * C::LDS_STRIDE + kk * C::Q + c * C::QK + 16 * v));
                acc[c * NBL + nb] = mfma32(afrag, bfrag, acc[c * NBL + nb]);
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // step 3: y[b][4*l + c]
    const int l = lt * 32 + ln;
#pragma unroll
    for (int nb = 0; nb < NBL; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t row = b0 + (nb0 + nb) * 32 + 8 * (i / 4) + 4 * g + (i % 4);
            if (row < B) {
                u32x2 v = {pack_bf16x2(acc[0 * NBL + nb][i], acc[1 * NBL + nb][i]),
                           pack_bf16x2(acc[2 * NBL + nb][i], acc[3 * NBL + nb][i])};
                *reinterpret_cast<u32x2*>(y + row * C::N_OUT + (size_t)l * K) = v;
            }
        }
}

template <typename C>
__global__ void __launch_bounds__(256)
fwd_wide_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ R,
                const uint16_t* __restrict__ L, uint16_t* __restrict__ y, int64_t B)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t y1s[];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, ln = lane & 31, g = lane >> 5;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;

    // ------------------------------------------------------------- stage 1 ----
    {
        const int kk = wave;
        const uint16_t* xrow[C::NB];
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) {
            int64_t row = b0 + nb * 32 + ln;
            row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
            xrow[nb] = x + row * C::N_IN + kk * C::P + 8 * g;
        }
        const uint16_t* Rk = R + ((size_t)kk * C::Q + ln) * C::P + 8 * g;
        constexpr int T = C::P / 16;
        for (int jg = 0; jg < C::QT / C::JG; ++jg) {
            f32x16 acc[C::JG * C::NB];
            zero_acc(acc);
            const uint16_t* Rg = Rk + (size_t)jg * C::JG * 32 * C::P;
            u32x4 xf[2][C::NB], rf[2][C::JG];
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb) xf[0][nb] = ldg128(xrow[nb]);
#pragma unroll
            for (int jj = 0; jj < C::JG; ++jj) rf[0][jj] = ldg128(Rg + (size_t)jj * 32 * C::P);
#pragma unroll 4
            for (int t = 0; t < T; ++t) {
                const int cur = t & 1, nxt = cur ^ 1;
                if (t + 1 < T) {
#pragma unroll
                    for (int nb = 0; nb < C::NB; ++nb) xf[nxt][nb] = ldg128(xrow[nb] + (t + 1) * 16);
#pragma unroll
                    for (int jj = 0; jj < C::JG; ++jj)
                        rf[nxt][jj] = ldg128(Rg + (size_t)jj * 32 * C::P + (t + 1) * 16);
                }
#pragma unroll
                for (int jj = 0; jj < C::JG; ++jj)
#pragma unroll
                    for (int nb = 0; nb < C::NB; ++nb)
                        acc[jj * C::NB + nb] =
                            mfma32(as_bf16x8(rf[cur][jj]), as_bf16x8(xf[cur][nb]), acc[jj * C::NB + nb]);
            }
            // lane holds D[j][b] for b = nb*32 + ln and j = jt*32 + 8*(i/4) + 4*g + i%4
#pragma unroll
            for (int jj = 0; jj < C::JG; ++jj)
#pragma unroll
                for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const f32x16& a = acc[jj * C::NB + nb];
                        u32x2 v = {pack_bf16x2(a[4 * i4 + 0], a[4 * i4 + 1]), pack_bf16x2(a[4 * i4 + 2], a[4 * i4 + 3])};
                        const int j = (jg * C::JG + jj) * 32 + 8 * i4 + 4 * g;
                        *reinterpret_cast<u32x2*>(y1s + (size_t)(nb * 32 + ln) * C::LDS_STRIDE + kk * C::Q + j) = v;
                    }
        }
    }
    __syncthreads();

    // ------------------------------------------------------------- stage 2 ----
    for (int rd = 0; rd < C::ROUNDS; ++rd)
        stage2_tile<C, C::NB>(L, y1s, y, b0, B, rd * 4 + wave, 0, ln, g);
    if constexpr (C::REM == 2) stage2_tile<C, 1>(L, y1s, y, b0, B, C::ROUNDS * 4 + (wave >> 1), wave & 1, ln, g);
}

template <typename C>
int launch(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    auto kern = fwd_wide_kernel<C>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
    if (e != hipSuccess) return -4;
    const int64_t grid = (pb.B + C::BM - 1) / C::BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), C::LDS_BYTES, st, (const uint16_t*)x,
                       (const uint16_t*)R, (const uint16_t*)L, (uint16_t*)y, pb.B);
    return hip_status(hipGetLastError());
}

struct Entry {
    int p, q, s;
    int (*fn)(const Problem&, const void*, const void*, const void*, void*, hipStream_t);
};

//                          P     Q     S    BM  JG
const Entry kTable[] = {
    {192, 192, 192, launch<FwdWide<192, 192, 192, 64, 6>>},   // ViT-B projection 768 -> 768
    {192, 192, 768, launch<FwdWide<192, 192, 768, 64, 6>>},   // GPT-2 small fc1 768 -> 3072
    {256, 256, 1024, launch<FwdWide<256, 256, 1024, 64, 4>>}, // GPT-2 medium fc1 1024 -> 4096
    {1024, 256, 256, launch<FwdWide<1024, 256, 256, 64, 4>>}, // GPT-2 medium fc2 4096 -> 1024
    {768, 192, 192, launch<FwdWide<768, 192, 192, 64, 6>>},   // GPT-2 small fc2 3072 -> 768
    {64, 64, 64, launch<FwdWide<64, 64, 64, 64, 2>>},         // small shapes (tests)
    {64, 64, 128, launch<FwdWide<64, 64, 128, 64, 2>>},
    {128, 64, 64, launch<FwdWide<128, 64, 64, 64, 2>>},
};

const Entry* find(const Problem& pb)
{
    if (pb.dtype != 1 || pb.k != 4 || pb.perm_b()) return nullptr;
    for (const Entry& e : kTable)
        if (e.p == pb.p && e.q == pb.q && e.s == pb.s) return &e;
    return nullptr;
}

}  // namespace

bool fwd_wide_supported(const Problem& pb) { return find(pb) != nullptr; }

int fwd_wide(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    const Entry* e = find(pb);
    return e ? e->fn(pb, x, R, L, y, st) : -2;
}

}  // namespace monarch
