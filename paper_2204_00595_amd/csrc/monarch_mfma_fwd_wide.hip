// Fused bf16 forward for "wide block" Monarch layers (k = 4 blocks, block sizes that are
// multiples of 32): both block-diagonal stages of Section 3.3 on v_mfma_f32_16x16x32_bf16,
// the mid permutation P^T folded into operand addressing, the intermediate in LDS only.
//
// One workgroup (4 waves) owns BM = 64 batch rows (four 16-row tiles).
//
// Why 16x16x32 and not 32x32x16: operands that come straight from global memory are loaded in
// MFMA layout, one row per lane group.  With 16-row tiles one load instruction covers 16 rows x
// 64 contiguous bytes, which the vector L1 serves at ~58 B/clk/CU on MI355X; the 32-row layout
// (32 rows x 32 bytes) is capped near 30 B/clk/CU (measured), and this kernel is bound by
// exactly that path: every workgroup streams all of R and L (0.6-2.6 MB) for its 64 rows.
//
// Stage 1  (step 1 of Section 3.3): wave w computes block kk = w,
//     Y1[b][kk][j] = sum_i R[kk][j][i] x[b][kk*P + i],
// as D^T = R . X^T so that each lane ends up with 4 consecutive j for one row b and writes
// them to LDS with one 8-byte store.  R and x fragments go global -> registers directly (every
// byte is needed by exactly one wave).  LDS holds Y1s[b][kk*Q + j] in bf16: the natural (k, q)
// grid, not permuted.
//
// Stage 2  (step 2): block c contracts over r = 0..Q-1 with
//     U[b][c*Q + r] = Y1[b][r % 4][c*Q/4 + r/4]      (P^T of Definition 3.1 on the (4, Q) grid).
// Which contraction index sits in which MFMA K-slot is free as long as both operands agree.
// Here a K-step covers 32 consecutive r (one 64-byte piece of an L row): lane group h takes the
// 16 bytes r = r0 + 8h .. +7, i.e. r1 = r0/4 + 2h + {0,1} for all four kk.  The matching
// activation operand is four 4-byte LDS reads (one per kk, two consecutive r1 each); the weight
// fragment is re-ordered to (kk, r1) slot order with four v_perm_b32.  No data is moved to apply
// the permutation.
// Waves split the output features l; each wave keeps all four c for its l-tiles so that step 3,
// y[b][4*l + c], becomes one packed 8-byte store per (b, l).
#include "monarch_internal.h"
#include "monarch_mfma_common.h"
#include <stdlib.h>

namespace monarch {

namespace {

template <int P_, int Q_, int S_, int JG_, int LT_, int R1_ = 3, int R2_ = 3, int DBG_ = 0>
struct FwdWide {
    static constexpr int K = 4, P = P_, Q = Q_, S = S_;
    static constexpr int BM = 64, NBT = 4;   // rows per workgroup, 16-row tiles
    static constexpr int JG = JG_;           // 16-wide j tiles a wave accumulates at once in stage 1
    static constexpr int LT = LT_;           // 16-wide l tiles a wave accumulates at once in stage 2
    static constexpr int R1 = R1_, R2 = R2_; // register-ring depths (K-steps in flight) of the stages
    static constexpr int DBG = DBG_;
    static constexpr int QK = Q / K;         // columns of each R block that feed one L block
    static constexpr int JT = Q / 16;        // j tiles per R block
    static constexpr int ST = S / 16;        // l tiles per L block
    static constexpr int KQ = K * Q;
    static constexpr int N_IN = K * P;
    static constexpr int N_OUT = K * S;
    static constexpr int LDS_STRIDE = KQ + 8;  // bf16; row stride = 4 dwords mod 64 banks
    static constexpr size_t LDS_BYTES = (size_t)BM * LDS_STRIDE * 2;
    static constexpr int T1 = P / 32;        // stage-1 K-steps per R block
    static constexpr int T2 = Q / 32;        // stage-2 K-steps per L block
    static_assert(P % 32 == 0 && Q % 32 == 0 && S % 16 == 0 && QK % 8 == 0, "tile shapes");
    static_assert(JT % JG == 0 && ST % (4 * LT) == 0, "tile groups");
    static_assert(T1 % R1 == 0 && R1 >= 2 && R2 >= 2, "ring depths");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

template <typename C>
__global__ void __launch_bounds__(256)
fwd_wide_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ R,
                const uint16_t* __restrict__ L, uint16_t* __restrict__ y, int64_t B)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t y1s[];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, l16 = lane & 15, h = lane >> 4;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;
    long long ts[4];
    if (C::DBG >= 4) ts[0] = __builtin_amdgcn_s_memtime();

    // ------------------------------------------------------------- stage 1 ----
    {
        const int kk = wave;
        const uint16_t* xrow[C::NBT];
#pragma unroll
        for (int bt = 0; bt < C::NBT; ++bt) {
            int64_t row = b0 + bt * 16 + l16;
            row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
            xrow[bt] = x + row * C::N_IN + kk * C::P + 8 * h;
        }
        const uint16_t* Rk = R + ((size_t)kk * C::Q + l16) * C::P + 8 * h;
        for (int jg = 0; jg < C::JT / C::JG; ++jg) {
            f32x4 acc[C::JG * C::NBT];
#pragma unroll
            for (int t = 0; t < C::JG * C::NBT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const uint16_t* Rg = Rk + (size_t)jg * C::JG * 16 * C::P;
            // register ring: K-step t + R1 - 1 is requested before the MFMAs of step t issue; the
            // scheduling barriers pin that order (the compiler otherwise sinks loads to their use)
            u32x4 xf[C::R1][C::NBT], rf[C::R1][C::JG];
            auto load_step = [&](int t, int slot) {
#pragma unroll
                for (int bt = 0; bt < C::NBT; ++bt) xf[slot][bt] = ldg128(xrow[bt] + t * 32);
#pragma unroll
                for (int jj = 0; jj < C::JG; ++jj) rf[slot][jj] = ldg128(Rg + (size_t)jj * 16 * C::P + t * 32);
            };
#pragma unroll
            for (int d = 0; d < C::R1 - 1; ++d) load_step(d, d);
            for (int t0 = 0; t0 < C::T1; t0 += C::R1) {
#pragma unroll
                for (int u = 0; u < C::R1; ++u) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (C::DBG != 6 && t0 + u + C::R1 - 1 < C::T1) load_step(t0 + u + C::R1 - 1, (u + C::R1 - 1) % C::R1);
                    __builtin_amdgcn_sched_barrier(0);
                    if (C::DBG == 5) {
#pragma unroll
                        for (int jj = 0; jj < C::JG; ++jj) acc[jj * C::NBT][0] += __uint_as_float(rf[u][jj][0] ^ rf[u][jj][3]);
#pragma unroll
                        for (int bt = 0; bt < C::NBT; ++bt) acc[bt][1] += __uint_as_float(xf[u][bt][0] ^ xf[u][bt][3]);
                        continue;
                    }
#pragma unroll
                    for (int jj = 0; jj < C::JG; ++jj)
#pragma unroll
                        for (int bt = 0; bt < C::NBT; ++bt)
                            acc[jj * C::NBT + bt] =
                                mfma16(as_bf16x8(rf[C::DBG == 6 ? 0 : u][jj]), as_bf16x8(xf[C::DBG == 6 ? 0 : u][bt]), acc[jj * C::NBT + bt]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // lane holds D^T[j][b] for b = bt*16 + l16 and j = jt*16 + 4*h + 0..3
#pragma unroll
            for (int jj = 0; jj < C::JG; ++jj)
#pragma unroll
                for (int bt = 0; bt < C::NBT; ++bt) {
                    const f32x4& a = acc[jj * C::NBT + bt];
                    const int j = (jg * C::JG + jj) * 16 + 4 * h;
                    *reinterpret_cast<u32x2*>(y1s + (size_t)(bt * 16 + l16) * C::LDS_STRIDE + kk * C::Q + j) =
                        u32x2{pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3])};
                }
        }
    }
    if (C::DBG >= 4) ts[1] = __builtin_amdgcn_s_memtime();
    __syncthreads();
    if (C::DBG >= 4) ts[2] = __builtin_amdgcn_s_memtime();

    // ------------------------------------------------------------- stage 2 ----
    // wave w owns l tiles (rd*4 + w)*LT .. +LT-1 in round rd
    for (int rd = 0; rd < C::ST / (4 * C::LT); ++rd) {
        const int lt0 = (rd * 4 + wave) * C::LT;
        f32x4 acc[C::K * C::LT * C::NBT];
#pragma unroll
        for (int t = 0; t < C::K * C::LT * C::NBT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        // L[c][l][r]: lane (l16, h) reads r = 32*t + 8*h .. +7 of row l = (lt0 + i)*16 + l16
        const uint16_t* Lbase = L + (size_t)(lt0 * 16 + l16) * C::Q + 8 * h;
        // Y1s[b][kk*Q + c*QK + r1], r1 = 8*t + 2*h + {0,1}: one dword per kk
        const uint16_t* abase = y1s + (size_t)l16 * C::LDS_STRIDE + 2 * h;

        constexpr int NSTEP = C::K * C::T2;  // (c, t) pairs
        u32x4 wf[C::R2][C::LT];
        u32x4 af[2][C::NBT];
        auto load_w = [&](int st, int slot) {
            const uint16_t* p = Lbase + (size_t)(st / C::T2) * C::S * C::Q + (st % C::T2) * 32;
#pragma unroll
            for (int i = 0; i < C::LT; ++i) wf[slot][i] = ldg128(p + (size_t)i * 16 * C::Q);
        };
        auto load_a = [&](int st, int slot) {
            const uint16_t* p = abase + (st / C::T2) * C::QK + (st % C::T2) * 8;
#pragma unroll
            for (int bt = 0; bt < C::NBT; ++bt)
#pragma unroll
                for (int kk = 0; kk < C::K; ++kk)
                    af[slot][bt][kk] = *reinterpret_cast<const uint32_t*>(p + (size_t)bt * 16 * C::LDS_STRIDE + kk * C::Q);
        };
#pragma unroll
        for (int d = 0; d < C::R2 - 1; ++d)
            if (d < NSTEP) load_w(d, d);
        load_a(0, 0);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            __builtin_amdgcn_sched_barrier(0);
            if (st + C::R2 - 1 < NSTEP) load_w(st + C::R2 - 1, (st + C::R2 - 1) % C::R2);
            if (st + 1 < NSTEP) load_a(st + 1, (st + 1) & 1);
            __builtin_amdgcn_sched_barrier(0);
            const int c = st / C::T2;
#pragma unroll
            for (int i = 0; i < C::LT; ++i) {
                // piece dwords: (r1a,k0 k1) (r1a,k2 k3) (r1b,k0 k1) (r1b,k2 k3) -> slots (kk, r1a r1b)
                const u32x4& p = wf[st % C::R2][i];
                const u32x4 wv = {pick_lo16(p[0], p[2]), pick_hi16(p[0], p[2]), pick_lo16(p[1], p[3]), pick_hi16(p[1], p[3])};
                const bf16x8 wfrag = as_bf16x8(wv);
#pragma unroll
                for (int bt = 0; bt < C::NBT; ++bt)
                    acc[(c * C::LT + i) * C::NBT + bt] =
                        mfma16(as_bf16x8(af[st & 1][bt]), wfrag, acc[(c * C::LT + i) * C::NBT + bt]);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // step 3: y[b][4*l + c]; lane holds D[b][l] for l = (lt0 + i)*16 + l16, b = bt*16 + 4*h + 0..3
#pragma unroll
        for (int i = 0; i < C::LT; ++i)
#pragma unroll
            for (int bt = 0; bt < C::NBT; ++bt)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t row = b0 + bt * 16 + 4 * h + e;
                    if (row < B) {
                        const int l = (lt0 + i) * 16 + l16;
                        u32x2 v = {pack_bf16x2(acc[(0 * C::LT + i) * C::NBT + bt][e], acc[(1 * C::LT + i) * C::NBT + bt][e]),
                                   pack_bf16x2(acc[(2 * C::LT + i) * C::NBT + bt][e], acc[(3 * C::LT + i) * C::NBT + bt][e])};
                        *reinterpret_cast<u32x2*>(y + row * C::N_OUT + (size_t)l * C::K) = v;
                    }
                }
    }
    if (C::DBG >= 4) {
        __builtin_amdgcn_s_waitcnt(0);
        ts[3] = __builtin_amdgcn_s_memtime();
        __syncthreads();
        if (lane == 0) {
            long long* o = reinterpret_cast<long long*>(y + b0 * C::N_OUT) + wave * 4;
            for (int i = 0; i < 4; ++i) o[i] = ts[i];
        }
    }
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
    int p, q, s, variant;
    int (*fn)(const Problem&, const void*, const void*, const void*, void*, hipStream_t);
};

// variant 0 is the default; the others are reachable with MONARCH_FWD_VARIANT=<n> (tuning aid)
//                                      P     Q     S   JG  LT  R1 R2
const Entry kTable[] = {
    {192, 192, 192, 0, launch<FwdWide<192, 192, 192, 12, 3, 3, 3>>},   // ViT-B projection 768 -> 768
    {192, 192, 192, 1, launch<FwdWide<192, 192, 192, 6, 3, 3, 3>>},
    {192, 192, 192, 2, launch<FwdWide<192, 192, 192, 6, 3, 3, 4>>},
    {192, 192, 192, 3, launch<FwdWide<192, 192, 192, 4, 3, 3, 4>>},
    {192, 192, 192, 11, launch<FwdWide<192, 192, 192, 12, 3, 3, 3, 4>>},
    {192, 192, 192, 12, launch<FwdWide<192, 192, 192, 12, 3, 3, 3, 5>>},
    {192, 192, 192, 13, launch<FwdWide<192, 192, 192, 12, 3, 3, 3, 6>>},
    {192, 192, 768, 0, launch<FwdWide<192, 192, 768, 12, 3, 3, 3>>},   // GPT-2 small fc1 768 -> 3072
    {192, 192, 768, 1, launch<FwdWide<192, 192, 768, 6, 3, 3, 4>>},
    {256, 256, 1024, 0, launch<FwdWide<256, 256, 1024, 8, 4, 4, 3>>},  // GPT-2 medium fc1 1024 -> 4096
    {256, 256, 1024, 1, launch<FwdWide<256, 256, 1024, 8, 2, 4, 4>>},
    {1024, 256, 256, 0, launch<FwdWide<1024, 256, 256, 8, 4, 4, 3>>},  // GPT-2 medium fc2 4096 -> 1024
    {1024, 256, 256, 1, launch<FwdWide<1024, 256, 256, 8, 4, 2, 3>>},
    {768, 192, 192, 0, launch<FwdWide<768, 192, 192, 12, 3, 3, 3>>},   // GPT-2 small fc2 3072 -> 768
    {64, 64, 64, 0, launch<FwdWide<64, 64, 64, 4, 1, 2, 3>>},          // small shapes (tests)
    {64, 64, 128, 0, launch<FwdWide<64, 64, 128, 4, 2, 2, 3>>},
    {128, 64, 64, 0, launch<FwdWide<128, 64, 64, 2, 1, 4, 3>>},
};

int tuning_variant()
{
    const char* v = getenv("MONARCH_FWD_VARIANT");
    return v ? atoi(v) : 0;
}

const Entry* find(const Problem& pb)
{
    if (pb.dtype != 1 || pb.k != 4 || pb.perm_b()) return nullptr;
    const int want = tuning_variant();
    const Entry* fallback = nullptr;
    for (const Entry& e : kTable)
        if (e.p == pb.p && e.q == pb.q && e.s == pb.s) {
            if (e.variant == want) return &e;
            if (e.variant == 0) fallback = &e;
        }
    return fallback;
}

}  // namespace

bool fwd_wide_supported(const Problem& pb) { return find(pb) != nullptr; }

int fwd_wide(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    const Entry* e = find(pb);
    return e ? e->fn(pb, x, R, L, y, st) : -2;
}

}  // namespace monarch
