// Fused bf16 forward for "wide block" Monarch layers (k = 4) with the weights pre-laid in MFMA
// fragment order (caller-provided workspace).  Both block-diagonal stages of Section 3.3 run on
// v_mfma_f32_32x32x16_bf16, the mid permutation P^T of Definition 3.1 is folded into the K-slot
// order of the packed L, the intermediate lives in LDS only.
//
// Why packed weights.  Every workgroup streams all of R and L; that stream is three quarters of
// the bytes a workgroup touches, and it bounds the kernel through the vector L1 (about 50-57 bytes
// per clock per CU when a wave instruction reads 1 KiB contiguously).  Staging row-major weights
// through LDS to transpose them into operand layout costs an LDS write plus an LDS read per byte
// on top, and LDS bandwidth then becomes the bound (measured: stage 2 of the LDS-staged kernel ran
// at a third of its L1 bound).  With the weights stored fragment by fragment, a weight operand is
// one fully coalesced 16-byte-per-lane global load straight into registers; LDS carries only the
// activations (x on the way in, the intermediate between the stages).
//
//   pack      (pack_fwd_kernel) one thread builds one 16-byte piece:
//             RF1[kk][t][jt][lane][e] = R[kk][32*jt + lane%32][16*t + 8*(lane/32) + e]
//             LF2[c][lt][ks][lane][e] = L[c][32*lt + lane%32][4*(4*ks + e%4) + 2*(lane/32) + e/4]
//   forward   one workgroup (4 waves) per 64 batch rows (two 32-row tiles):
//     stage 1 (step 1): wave w computes block kk = w, D^T = R[kk] . X^T, all Q columns in
//             accumulators.  x arrives through a wave-private LDS ring of 64-column chunks filled by
//             global_load_lds_dwordx4 in full 128-byte lines (two chunks ahead: HBM latency); the
//             R fragments arrive in a register ring three K-steps ahead (L2 latency).
//     Y1      is written to LDS as Y1s[b][j/4][kk][j%4] (bf16): the 32 bytes of block j/4 hold, for
//             four consecutive j, all four kk.
//     stage 2 (step 2): U[b][c*Q + r] = Y1[b][r%4][c*Q/4 + r/4] (P^T on the (4, Q) grid), so K-step
//             ks of block c is exactly LDS block c*Q/16 + ks: lane group g reads its 16-byte half
//             (kk = 2g, 2g+1; four j each) with one ds_read_b128, and LF2 holds L's columns in the
//             matching slot order.  No instruction is spent on the permutation.
//             Work is split over waves in units of (32 features l) x (32 rows); a wave keeps all four
//             c of its units so that step 3, y[b][4*l + c], is one packed 8-byte store per (b, l).
#include "monarch_internal.h"
#include "monarch_mfma_common.h"
#include "monarch_mfma_stage1.h"
#include "monarch_act.h"

namespace monarch {

namespace {

// ------------------------------------------------------------------------ pack ----

__global__ void __launch_bounds__(256)
pack_fwd_kernel(const uint16_t* __restrict__ R, const uint16_t* __restrict__ L, uint16_t* __restrict__ RF1,
                uint16_t* __restrict__ LF2, int P, int Q, int S)
{
    const int nR = 4 * Q * P / 8, nL = 4 * S * Q / 8;  // 16-byte pieces per array
    int pc = blockIdx.x * 256 + threadIdx.x;
    if (pc < nR) {
        const int lane = pc & 63;
        int rest = pc >> 6;
        const int QT = Q / 32, T = P / 16;
        const int jt = rest % QT; rest /= QT;
        const int t = rest % T;
        const int kk = rest / T;
        const uint16_t* src = R + ((size_t)kk * Q + 32 * jt + (lane & 31)) * P + 16 * t + 8 * (lane >> 5);
        *reinterpret_cast<u32x4*>(RF1 + (size_t)pc * 8) = *reinterpret_cast<const u32x4*>(src);
    } else if (pc < nR + nL) {
        pc -= nR;
        const int lane = pc & 63;
        int rest = pc >> 6;
        const int KS = Q / 16, NLT = S / 32;
        const int ks = rest % KS; rest /= KS;
        const int lt = rest % NLT;
        const int c = rest / NLT;
        const int g = lane >> 5;
        const uint16_t* src = L + ((size_t)c * S + 32 * lt + (lane & 31)) * Q + 16 * ks;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = src[4 * (e & 3) + 2 * g + (e >> 2)];
        u32x4 o;
#pragma unroll
        for (int w = 0; w < 4; ++w) o[w] = (uint32_t)v[2 * w] | ((uint32_t)v[2 * w + 1] << 16);
        *reinterpret_cast<u32x4*>(LF2 + (size_t)pc * 8) = o;
    }
}

// --------------------------------------------------------------------- forward ----

template <int P_, int Q_, int S_, int UPW_, int RW2_>
struct FwdFrag {
    static constexpr int K = 4, P = P_, Q = Q_, S = S_;
    static constexpr int BM = 64, NB = 2;     // rows per workgroup, 32-row tiles
    static constexpr int UPW = UPW_;          // stage-2 units (32 l x 32 rows) per wave per pass
    static constexpr int RW2 = RW2_;          // stage-2 weight ring, K-steps
    static constexpr int QT = Q / 32;         // 32-wide j tiles per R block
    static constexpr int KQ = K * Q;
    static constexpr int N_IN = K * P, N_OUT = K * S;
    using S1 = Stage1<P_, Q_>;
    static constexpr int XR = S1::XR;
    static constexpr int KS = Q / 16;         // stage-2 K-steps per L block
    static constexpr int NLT_ALL = S / 32;
    static constexpr int UNITS = NLT_ALL * NB;
    static constexpr int PASSES = UNITS / (4 * UPW);
    static constexpr int NLT = (UPW + 1) / 2; // l tiles a wave touches in one pass
    static constexpr int Y1_STRIDE = KQ + 8;  // bf16; row stride = 4 dwords mod 64 banks
    static constexpr size_t LDS_Y1 = (size_t)BM * Y1_STRIDE * 2;
    static constexpr size_t LDS_X = S1::LDS_X;
    static constexpr size_t LDS_BYTES = LDS_Y1 > LDS_X ? LDS_Y1 : LDS_X;
    static_assert(P % 64 == 0 && Q % 32 == 0 && S % 32 == 0 && Q % 16 == 0, "tile shapes");
    static_assert(UNITS % (4 * UPW) == 0 && UPW >= 1 && UPW <= 4, "stage-2 split");
    static_assert(KS % RW2 == 0 && RW2 % 2 == 0 && RW2 >= 2, "stage-2 ring");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

// Base pointers of the packed L fragments a wave streams in the stage-2 pass that starts at work unit u0:
// fragment (c, lt, ks) sits at ((c*NLT_ALL + lt)*KS + ks) * 512 elements, + lane * 8.
template <typename C>
__device__ __forceinline__ void stage2_wbase(const uint16_t* __restrict__ LF2, int u0, int lane, const uint16_t* (&wbase)[C::NLT])
{
    const int lt_lo = u0 >> 1;
    // the second l tile may not exist for the last wave (its units then never use it): reuse the first
    const int lt_hi = (lt_lo + 1 < C::NLT_ALL) ? lt_lo + 1 : lt_lo;
    wbase[0] = LF2 + ((size_t)lt_lo * C::KS * 64 + lane) * 8;
    if (C::NLT > 1) wbase[C::NLT - 1] = LF2 + ((size_t)lt_hi * C::KS * 64 + lane) * 8;
}

// weights of K-step (c, ks) into ring slot `slot`
template <typename C>
__device__ __forceinline__ void stage2_issue_w(const uint16_t* const (&wbase)[C::NLT], u32x4 (&wr)[C::RW2][C::NLT], int c, int ks, int slot)
{
#pragma unroll
    for (int li = 0; li < C::NLT; ++li)
        wr[slot][li] = ldg128(wbase[li] + ((size_t)c * C::NLT_ALL * C::KS + ks) * 512);
}

// One stage-2 pass of one wave: work units u0 .. u0+UPW-1, unit w = (l tile w / 2, row tile w % 2).
// PRE: the caller has already issued the weights of steps 0 .. RW-2 into `wr` (first pass: they
// are fetched while the workgroup is still exchanging Y1 through LDS).
// BIAS: the bias (when the pointer is not null) is added to the product.  ACT: the sum also goes to y_pre
// (when not null) and y receives gelu of it.
template <typename C, bool ODD, bool PRE, bool BIAS, bool ACT>
__device__ __forceinline__ void stage2_pass(const uint16_t* __restrict__ LF2, const uint16_t* y1s,
                                            const uint16_t* __restrict__ bias, uint16_t* __restrict__ y,
                                            uint16_t* __restrict__ y_pre, int64_t b0,
                                            int64_t B, int u0, int lane, u32x4 (&wr)[C::RW2][C::NLT])
{
    constexpr int UPW = C::UPW, K = 4, NLT = C::NLT, RW = C::RW2, KS = C::KS;
    constexpr int NSTEP = K * KS;  // flat K-steps n = c*KS + ks; the activation block of step n is LDS block n
    const int ln = lane & 31, g = lane >> 5;
    const int lt_lo = u0 >> 1;
    const uint16_t* wbase[NLT];
    stage2_wbase<C>(LF2, u0, lane, wbase);
    const uint16_t* abase = y1s + (size_t)ln * C::Y1_STRIDE + 8 * g;

    f32x16 acc[UPW * K];
#pragma unroll
    for (int t = 0; t < UPW * K; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    u32x4 ar[2][C::NB];
    auto issue_w = [&](int c, int ks, int slot) { stage2_issue_w<C>(wbase, wr, c, ks, slot); };
    auto read_a = [&](int n, int slot) {
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) ar[slot][nb] = lds128(abase + (size_t)nb * 32 * C::Y1_STRIDE + n * 16);
    };
    // prologue: weights of steps 0 .. RW-2, activations of step 0
    if (!PRE) {
#pragma unroll
        for (int d = 0; d < RW - 1; ++d) issue_w(d / KS, d % KS, d);
    }
    read_a(0, 0);
#pragma unroll
    for (int c = 0; c < K; ++c) {
        for (int kg = 0; kg < KS; kg += RW) {
#pragma unroll
            for (int kr = 0; kr < RW; ++kr) {
                const int ks = kg + kr, n = c * KS + ks;
                __builtin_amdgcn_sched_barrier(0);
                {
                    // step n + RW - 1 goes to the slot step n - 1 has just left
                    const int ksn = ks + RW - 1;
                    const int cn = c + ksn / KS;
                    if (cn < K) issue_w(cn, ksn % KS, (kr + RW - 1) % RW);
                }
                if (n + 1 < NSTEP) read_a(n + 1, (kr + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < UPW; ++i) {
                    const int ww = i + (ODD ? 1 : 0);  // work unit relative to the first l tile
                    acc[i * K + c] = mfma32(as_bf16x8(ar[kr & 1][ww & 1]), as_bf16x8(wr[kr][ww >> 1]), acc[i * K + c]);
                }
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // step 3: y[b][4*l + c]; lane holds D[b][l] for l = lt*32 + ln, b = nb*32 + 8*(i/4) + 4*g + i%4
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
        const int ww = i + (ODD ? 1 : 0);
        const int l = (lt_lo + (ww >> 1)) * 32 + ln;
        float bv[K] = {0.f, 0.f, 0.f, 0.f};
        if (BIAS && bias) {
            // the lane's four outputs of a row are y[row][4*l .. 4*l+3]: one 8-byte piece of the bias
            const u32x2 bb = *reinterpret_cast<const u32x2*>(bias + (size_t)l * K);
            bv[0] = __uint_as_float(bb[0] << 16), bv[1] = __uint_as_float(bb[0] & 0xffff0000u);
            bv[2] = __uint_as_float(bb[1] << 16), bv[3] = __uint_as_float(bb[1] & 0xffff0000u);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t row = b0 + (ww & 1) * 32 + 8 * (e / 4) + 4 * g + (e % 4);
            if (row < B) {
                float o[K] = {acc[i * K + 0][e], acc[i * K + 1][e], acc[i * K + 2][e], acc[i * K + 3][e]};
                if constexpr (BIAS) {
#pragma unroll
                    for (int c = 0; c < K; ++c) o[c] += bv[c];
                }
                if constexpr (ACT) {
                    if (y_pre) {
                        u32x2 h = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
                        __builtin_nontemporal_store(h, reinterpret_cast<u32x2*>(y_pre + row * C::N_OUT + (size_t)l * K));
                    }
#pragma unroll
                    for (int c = 0; c < K; ++c) o[c] = gelu_f(o[c]);
                }
                u32x2 v = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
                __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(y + row * C::N_OUT + (size_t)l * K));
            }
        }
    }
}

template <typename C, bool BIAS, bool ACT>
__global__ void __launch_bounds__(256)
fwd_frag_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ RF1,
                const uint16_t* __restrict__ LF2, const uint16_t* __restrict__ bias, uint16_t* __restrict__ y,
                uint16_t* __restrict__ y_pre, int64_t B)
{
    extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 31, g = lane >> 5;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;

    u32x4 wr2[C::RW2][C::NLT];  // stage-2 weight ring
    // Short batches leave CUs without a row tile: gridDim.y workgroups then share a row tile, each taking a
    // contiguous share of the stage-2 passes (its own columns of y, its own part of the L stream) after computing
    // stage 1 for itself.
    const int ps_lo = (int)blockIdx.y * C::PASSES / (int)gridDim.y, ps_hi = ((int)blockIdx.y + 1) * C::PASSES / (int)gridDim.y;
    // ------------------------------------------------------------- stage 1 ----
    {
        const int kk = wave;
        f32x16 acc[C::QT * C::NB];
        stage1_block<typename C::S1>(x, RF1, b0, B, kk, lane, lds + (size_t)wave * C::XR * 4096, acc);
        __builtin_amdgcn_sched_barrier(0);
        {
            // the first stage-2 weights travel while the workgroup exchanges Y1 through LDS
            const uint16_t* wbase[C::NLT];
            stage2_wbase<C>(LF2, (ps_lo * 4 + wave) * C::UPW, lane, wbase);
#pragma unroll
            for (int d = 0; d < C::RW2 - 1; ++d) stage2_issue_w<C>(wbase, wr2, d / C::KS, d % C::KS, d);
        }
        __syncthreads();  // every wave is done with its x ring: the space becomes Y1s
        // lane holds D^T[j][b] for b = nb*32 + ln and j = jt*32 + 8*(i/4) + 4*g + i%4
#pragma unroll
        for (int jt = 0; jt < C::QT; ++jt)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x16& a = acc[jt * C::NB + nb];
                    const int j = jt * 32 + 8 * i4 + 4 * g;  // four consecutive j: one 8-byte slot of block j/4
                    *reinterpret_cast<u32x2*>(lds + (size_t)(nb * 32 + ln) * C::Y1_STRIDE + (j >> 2) * 16 + kk * 4) =
                        u32x2{pack_bf16x2(a[4 * i4 + 0], a[4 * i4 + 1]), pack_bf16x2(a[4 * i4 + 2], a[4 * i4 + 3])};
                }
    }
    __syncthreads();

    // ------------------------------------------------------------- stage 2 ----
    {
        const int u0 = (ps_lo * 4 + wave) * C::UPW;
        if (u0 & 1)
            stage2_pass<C, true, true, BIAS, ACT>(LF2, lds, bias, y, y_pre, b0, B, u0, lane, wr2);
        else
            stage2_pass<C, false, true, BIAS, ACT>(LF2, lds, bias, y, y_pre, b0, B, u0, lane, wr2);
    }
    for (int ps = ps_lo + 1; ps < ps_hi; ++ps) {
        const int u0 = (ps * 4 + wave) * C::UPW;
        if (u0 & 1)
            stage2_pass<C, true, false, BIAS, ACT>(LF2, lds, bias, y, y_pre, b0, B, u0, lane, wr2);
        else
            stage2_pass<C, false, false, BIAS, ACT>(LF2, lds, bias, y, y_pre, b0, B, u0, lane, wr2);
    }
}

// ---- eight waves per workgroup (two per SIMD) for the shapes with 256-wide blocks ----
// Same tiling of the work (64 rows per workgroup, all of R and L streamed once per workgroup), but each
// block of stage 1 is shared by two waves (column halves, stage1_half) and stage 2 runs eight waves on
// units of one l tile x two row tiles: half the accumulators per wave, so two waves fit a SIMD and one
// computes while the other waits for its weight fragments.
// PRIV: every wave keeps an x ring of its own (two slots; x passes through the L1 twice, no barriers in
// stage 1) instead of sharing one with its partner (stage1_half: one barrier per 64-column chunk).
template <int P_, int Q_, int S_, int RW2_, bool PRIV_>
struct FwdFrag8 {
    static constexpr int K = 4, P = P_, Q = Q_, S = S_;
    static constexpr int BM = 64, NB = 2, NW = 8;
    static constexpr int UPW = 2;             // one l tile, both row tiles
    static constexpr int RW2 = RW2_;
    static constexpr int QT = Q / 32, QH = QT / 2;
    static constexpr int KQ = K * Q;
    static constexpr int N_IN = K * P, N_OUT = K * S;
    static constexpr bool PRIV = PRIV_;
    using S1 = Stage1<P_, Q_>;                        // shared ring: the pair's columns together
    using S1P = Stage1<P_, Q_ / 2, Q_ / 32, 2>;       // private rings: this wave's half of the columns
    static constexpr int XR = PRIV ? S1P::XR : 3;
    static constexpr int KS = Q / 16;
    static constexpr int NLT_ALL = S / 32;
    static constexpr int UNITS = NLT_ALL * NB;
    static constexpr int PASSES = UNITS / (NW * UPW);
    static constexpr int NLT = 1;
    static constexpr int Y1_STRIDE = KQ + 8;
    static constexpr size_t LDS_Y1 = (size_t)BM * Y1_STRIDE * 2;
    static constexpr size_t LDS_X = (size_t)(PRIV ? 8 : 4) * XR * 8192;  // one ring per wave / per pair of waves
    static constexpr size_t LDS_BYTES = LDS_Y1 > LDS_X ? LDS_Y1 : LDS_X;
    static_assert(P % 64 == 0 && P / 64 >= XR && Q % 64 == 0 && S % 32 == 0, "tile shapes");
    static_assert(UNITS % (NW * UPW) == 0, "stage-2 split");
    static_assert(KS % RW2 == 0 && RW2 % 2 == 0 && RW2 >= 2, "stage-2 ring");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

template <typename C, bool BIAS, bool ACT>
__global__ void __launch_bounds__(512)
fwd_frag8_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ RF1,
                 const uint16_t* __restrict__ LF2, const uint16_t* __restrict__ bias, uint16_t* __restrict__ y,
                 uint16_t* __restrict__ y_pre, int64_t B)
{
    extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 31, g = lane >> 5;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;

    u32x4 wr2[C::RW2][C::NLT];  // stage-2 weight ring
    // gridDim.y workgroups share a row tile, each with a contiguous share of the stage-2 passes (see fwd_frag_kernel)
    const int ps_lo = (int)blockIdx.y * C::PASSES / (int)gridDim.y, ps_hi = ((int)blockIdx.y + 1) * C::PASSES / (int)gridDim.y;
    {
        const int kk = wave & 3, half = wave >> 2;
        f32x16 acc[C::QH * C::NB];
        if constexpr (C::PRIV)
            stage1_block<typename C::S1P>(x, RF1, b0, B, kk, lane, lds + (size_t)wave * C::XR * 4096, acc, half * C::QH);
        else
            stage1_half<typename C::S1>(x, RF1, b0, B, kk, half, lane, lds + (size_t)kk * C::XR * 4096, acc);
        __builtin_amdgcn_sched_barrier(0);
        {
            const uint16_t* wbase[C::NLT];
            stage2_wbase<C>(LF2, (ps_lo * C::NW + wave) * C::UPW, lane, wbase);
#pragma unroll
            for (int d = 0; d < C::RW2 - 1; ++d) stage2_issue_w<C>(wbase, wr2, d / C::KS, d % C::KS, d);
        }
        __syncthreads();  // every wave is done with the x rings: the space becomes Y1s
#pragma unroll
        for (int jl = 0; jl < C::QH; ++jl)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const f32x16& a = acc[jl * C::NB + nb];
                    const int j = (half * C::QH + jl) * 32 + 8 * i4 + 4 * g;
                    *reinterpret_cast<u32x2*>(lds + (size_t)(nb * 32 + ln) * C::Y1_STRIDE + (j >> 2) * 16 + kk * 4) =
                        u32x2{pack_bf16x2(a[4 * i4 + 0], a[4 * i4 + 1]), pack_bf16x2(a[4 * i4 + 2], a[4 * i4 + 3])};
                }
    }
    __syncthreads();
    stage2_pass<C, false, true, BIAS, ACT>(LF2, lds, bias, y, y_pre, b0, B, (ps_lo * C::NW + wave) * C::UPW, lane, wr2);
    for (int ps = ps_lo + 1; ps < ps_hi; ++ps)
        stage2_pass<C, false, false, BIAS, ACT>(LF2, lds, bias, y, y_pre, b0, B, (ps * C::NW + wave) * C::UPW, lane, wr2);
}

template <typename C>
int launch8(const Problem& pb, const void* x, const uint16_t* RF1, const uint16_t* LF2, void* y, hipStream_t st)
{
    auto kern = pb.act ? fwd_frag8_kernel<C, true, true> : (pb.bias ? fwd_frag8_kernel<C, true, false> : fwd_frag8_kernel<C, false, false>);
    hipError_t e = allow_dynamic_lds((const void*)kern, C::LDS_BYTES);
    if (e != hipSuccess) return -4;
    const int64_t grid = (pb.B + C::BM - 1) / C::BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid, (unsigned)pass_split(grid, C::PASSES)), dim3(512), C::LDS_BYTES, st, (const uint16_t*)x, RF1, LF2,
                       (const uint16_t*)pb.bias, (uint16_t*)y, (uint16_t*)pb.y_pre, pb.B);
    return hip_status(hipGetLastError());
}

template <typename C>
int launch(const Problem& pb, const void* x, const uint16_t* RF1, const uint16_t* LF2, void* y, hipStream_t st)
{
    // with the nonlinearity the bias pointer is tested inside the kernel (one variant for both cases)
    auto kern = pb.act ? fwd_frag_kernel<C, true, true> : (pb.bias ? fwd_frag_kernel<C, true, false> : fwd_frag_kernel<C, false, false>);
    hipError_t e = allow_dynamic_lds((const void*)kern, C::LDS_BYTES);
    if (e != hipSuccess) return -4;
    const int64_t grid = (pb.B + C::BM - 1) / C::BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid, (unsigned)pass_split(grid, C::PASSES)), dim3(256), C::LDS_BYTES, st, (const uint16_t*)x, RF1, LF2,
                       (const uint16_t*)pb.bias, (uint16_t*)y, (uint16_t*)pb.y_pre, pb.B);
    return hip_status(hipGetLastError());
}

struct Entry {
    int p, q, s;
    int (*fn)(const Problem&, const void*, const uint16_t*, const uint16_t*, void*, hipStream_t);
};

//                                 P     Q     S  UPW RW2
const Entry kTable[] = {
    {192, 192, 192, launch<FwdFrag<192, 192, 192, 3, 6>>},    // ViT-B projection 768 -> 768
    {192, 192, 768, launch8<FwdFrag8<192, 192, 768, 6, false>>},    // GPT-2 small fc1 768 -> 3072
    {256, 256, 1024, launch8<FwdFrag8<256, 256, 1024, 8, false>>},  // GPT-2 medium fc1 1024 -> 4096
    {1024, 256, 256, launch<FwdFrag<1024, 256, 256, 4, 8>>},  // GPT-2 medium fc2 4096 -> 1024
    {768, 192, 192, launch<FwdFrag<768, 192, 192, 3, 6>>},    // GPT-2 small fc2 3072 -> 768
    {256, 256, 256, launch8<FwdFrag8<256, 256, 256, 8, false>>},    // GPT-2 medium projection 1024 -> 1024
    {192, 192, 576, launch<FwdFrag<192, 192, 576, 3, 6>>},    // ViT-B / GPT-2 small fused q,k,v 768 -> 2304
    {256, 256, 768, launch8<FwdFrag8<256, 256, 768, 8, false>>},    // GPT-2 medium fused q,k,v 1024 -> 3072
    {128, 128, 128, launch<FwdFrag<128, 128, 128, 2, 4>>},    // width 512 (MLP-Mixer-S): 512 -> 512
    {128, 128, 512, launch<FwdFrag<128, 128, 512, 4, 4>>},    // 512 -> 2048
    {512, 128, 128, launch<FwdFrag<512, 128, 128, 2, 4>>},    // 2048 -> 512
    {64, 64, 64, launch<FwdFrag<64, 64, 64, 1, 4>>},          // small shapes (tests)
    {64, 64, 128, launch<FwdFrag<64, 64, 128, 2, 4>>},
    {128, 64, 64, launch<FwdFrag<128, 64, 64, 1, 4>>},
};

const Entry* find(const Problem& pb)
{
    if (pb.dtype != 1 || pb.k != 4 || pb.perm_b()) return nullptr;
    for (const Entry& e : kTable)
        if (e.p == pb.p && e.q == pb.q && e.s == pb.s) return &e;
    return nullptr;
}

}  // namespace

bool fwd_frag_supported(const Problem& pb) { return find(pb) != nullptr; }

// packed R then packed L, each the size of its source
size_t fwd_frag_workspace(const Problem& pb) { return align_up(pb.n_R() * 2, 256) + align_up(pb.n_L() * 2, 256); }

int fwd_frag(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    const Entry* e = find(pb);
    if (!e) return -2;
    uint16_t* RF1 = (uint16_t*)ws;
    uint16_t* LF2 = (uint16_t*)((char*)ws + align_up(pb.n_R() * 2, 256));
    if (!pb.ws_packed()) {
        const size_t pieces = (pb.n_R() + pb.n_L()) / 8;
        hipLaunchKernelGGL(pack_fwd_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st,
                           (const uint16_t*)R, (const uint16_t*)L, RF1, LF2, pb.p, pb.q, pb.s);
        if (hipGetLastError() != hipSuccess) return -4;
    }
    return e->fn(pb, x, RF1, LF2, y, st);
}

}  // namespace monarch
