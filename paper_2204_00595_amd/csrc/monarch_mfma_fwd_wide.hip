// Fused bf16 forward for "wide block" Monarch layers (k = 4 blocks, block sizes that are
// multiples of 32): both block-diagonal stages of Section 3.3 on v_mfma_f32_32x32x16_bf16,
// the mid permutation P^T folded into operand addressing, the intermediate in LDS only.
//
// One workgroup (4 waves) owns BM = 64 batch rows (two 32-row tiles).
//
// Data movement.  Every workgroup streams all of R and L (0.6-2.6 MB) plus its rows of x through
// the vector L1, and that path is what bounds the kernel.  The L1 serves about one cache-line
// access per clock, so operands are fetched with adjacent lanes on adjacent 16-byte pieces
// (16 rows x 64 contiguous bytes per instruction = full rate) and written straight into LDS
// (global_load_lds_dwordx4, no VGPR staging); the MFMA fragments are then read back from LDS in
// operand layout (row = lane % 32).  Loading fragments directly from global in operand layout
// touches 64 lines per instruction and runs at a quarter of that rate (measured).
// LDS staging blocks are 16 rows x 64 bytes = 1 KiB; the four 16-byte pieces of a row are stored
// XOR-swizzled with bits 2..3 of the row so that ds_read_b128 of a fragment is conflict-free.
//
// Stage 1  (step 1 of Section 3.3): wave w computes block kk = w,
//     Y1[b][kk][j] = sum_i R[kk][j][i] x[b][kk*P + i],
// as D^T = R . X^T, accumulating all Q columns in registers while its private LDS ring holds
// 32-column chunks of R[kk] and x.  When every wave is done the staging space is recycled:
// Y1 is written to LDS as Y1s[b][kk*Q + j] in bf16 (8-byte stores, natural (k, q) grid).
//
// Stage 2  (step 2): block c contracts over r = 0..Q-1 with
//     U[b][c*Q + r] = Y1[b][r % 4][c*Q/4 + r/4]      (P^T of Definition 3.1 on the (4, Q) grid).
// Which contraction index sits in which MFMA K-slot is free as long as both operands agree.
// A K-step covers 16 consecutive r of an L row; lane group g takes the 16 bytes r = r0 + 8g .. +7,
// i.e. r1 = r0/4 + 2g + {0,1} for all four kk.  The matching activation operand is four 4-byte LDS
// reads of Y1s (one per kk); the weight fragment is re-ordered to (kk, r1) slot order with four
// v_perm_b32.  No data is moved to apply the permutation.
// Work is split over waves in units of (32 features l) x (32 rows); every wave keeps all four c of
// its units so that step 3, y[b][4*l + c], is one packed 8-byte store per (b, l).
#include "monarch_internal.h"
#include "monarch_mfma_common.h"

namespace monarch {

namespace {

template <int P_, int Q_, int S_, int UPW_, int D2_ = 3, int RD1_ = 8>
struct FwdWide {
    static constexpr int K = 4, P = P_, Q = Q_, S = S_;
    static constexpr int BM = 64, NB = 2;     // rows per workgroup, 32-row tiles
    static constexpr int UPW = UPW_;          // stage-2 units (32 l x 32 rows) per wave per pass
    static constexpr int RD1 = RD1_;          // stage-1 LDS ring: 4 KiB units (32 rows x 128 bytes)
    static constexpr int D2 = D2_;            // stage-2 LDS ring depth (chunks, or 4 KiB units)
    static constexpr int QK = Q / K;          // columns of each R block that feed one L block
    static constexpr int QT = Q / 32;         // 32-wide j tiles per R block
    static constexpr int KQ = K * Q;
    static constexpr int N_IN = K * P, N_OUT = K * S;
    static constexpr int C1 = P / 64;         // stage-1 column chunks (one 128-byte line of R / x per row)
    static constexpr int UPC = QT + 2;        // stage-1 units per chunk: two x units, then the R tiles
    static constexpr int NU1 = C1 * UPC;
    static constexpr int TQ = Q / 32;         // stage-2 chunks per L block (32 columns of L each)
    static constexpr int UNITS = (S / 32) * NB;
    static constexpr int PASSES = UNITS / (4 * UPW);
    static constexpr int NLT = (UPW + 1) / 2; // l tiles a wave touches in one pass
    static constexpr int NBLK2 = 2 * NLT;     // staging blocks per stage-2 chunk
    static constexpr int Y1_STRIDE = KQ + 8;  // bf16; row stride = 4 dwords mod 64 banks (16-byte reads, row = lane)
    static constexpr size_t LDS_Y1 = ((size_t)BM * Y1_STRIDE * 2 + 1023) / 1024 * 1024;
    static constexpr size_t STG1 = (size_t)RD1 * 4096;         // per wave
    // stage 2 streams L in 4 KiB units of full 128-byte lines when the ring fits beside Y1s,
    // else in 32-column chunks (64 bytes per row)
    static constexpr bool S2_LINES = (Q % 64 == 0) && (LDS_Y1 + 4 * (size_t)D2 * 4096 <= kMaxLdsBytes);
    static constexpr size_t STG2 = S2_LINES ? (size_t)D2 * 4096 : (size_t)D2 * NBLK2 * 1024;  // per wave
    static constexpr size_t LDS_S1 = 4 * STG1, LDS_S2 = LDS_Y1 + 4 * STG2;
    static constexpr size_t LDS_BYTES = LDS_S1 > LDS_S2 ? LDS_S1 : LDS_S2;
    static_assert(P % 64 == 0 && Q % 32 == 0 && S % 32 == 0 && QK % 8 == 0, "tile shapes");
    static_assert(QT % 2 == 0 && RD1 >= 3 && (RD1 - 2) * 4 < 64, "stage-1 stream");
    static_assert(UNITS % (4 * UPW) == 0 && UPW >= 1 && UPW <= 4, "stage-2 split");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt = simm16[3:0] | simm16[15:14] << 4)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// one global_load_lds_dwordx4: every lane fetches 16 bytes from its own address, the wave's 1 KiB
// lands contiguously at `lds_block` (+ lane * 16)
__device__ __forceinline__ void dma16(const uint16_t* gsrc, uint16_t* lds_block)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                     (__attribute__((address_space(3))) void*)lds_block, 16, 0, 0);
}

// vmcnt(4 * units) for a unit count known after unrolling (a unit = four DMA instructions)
__device__ __forceinline__ void wait_vmcnt_units(int units)
{
    switch (units) {
        case 0: wait_vmcnt<0>(); break;
        case 1: wait_vmcnt<4>(); break;
        case 2: wait_vmcnt<8>(); break;
        case 3: wait_vmcnt<12>(); break;
        case 4: wait_vmcnt<16>(); break;
        case 5: wait_vmcnt<20>(); break;
        case 6: wait_vmcnt<24>(); break;
        case 7: wait_vmcnt<28>(); break;
        default: wait_vmcnt<32>(); break;
    }
}

__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// 4 KiB staging unit = 32 rows x 128 bytes = four 1 KiB blocks of 8 rows.  One DMA instruction
// fills a block: lane s fetches row s/8, and its slot s%8 holds logical 16-byte piece
// (s%8) ^ key, key = (row & 7) ^ ((row >> 3) & 1), which makes the fragment reads conflict-free.
// A fragment for K-step u (16 columns) is pieces 2u and 2u+1: lane (row = lane%32, g = lane/32).
__device__ __forceinline__ int unit_frag_off(int ln, int g, int u)
{
    const int bi = ln >> 3, r = ln & 7;
    return bi * 512 + r * 64 + 8 * ((2 * u + g) ^ r ^ (bi & 1));
}

// same, for an explicit 16-byte piece index (0..7) of the row
__device__ __forceinline__ int unit_piece_off(int ln, int piece)
{
    const int bi = ln >> 3, r = ln & 7;
    return bi * 512 + r * 64 + 8 * (piece ^ r ^ (bi & 1));
}

// Stage 2 on full-line units (Q % 64 == 0 and room for the ring).  One pass of one wave:
// work units u0 .. u0+UPW-1, work unit w = (l tile w / 2, row tile w % 2).
template <typename C, bool ODD>
__device__ __forceinline__ void stage2_pass_lines(const uint16_t* __restrict__ L, const uint16_t* y1s, uint16_t* stg,
                                                  uint16_t* __restrict__ y, int64_t b0, int64_t B, int u0, int lane)
{
    constexpr int UPW = C::UPW, K = 4, NLT = C::NLT, RD = C::D2;
    constexpr int TQ64 = C::Q / 64;
    constexpr int NU = K * TQ64 * NLT;  // staged units, in (c, tq, li) order
    const int ln = lane & 31, g = lane >> 5;
    const int lt_lo = u0 >> 1;
    const int rb = lane >> 3, pe = (lane & 7) ^ rb;  // DMA: row in block, logical piece for even blocks
    // rows of the staged l tiles (the second tile may not exist for the last wave: reuse the first)
    const bool second_ok = (lt_lo + 1) * 32 < C::S;
    const uint16_t* Lrow = L + ((size_t)lt_lo * 32 + rb) * C::Q;
    // K-step (pp, m) of a unit: lane group g contracts over the 8 r = 16*(2pp + g) + 8m .. +7 of the
    // unit's 64, i.e. half m of the 32-byte block 2pp + g of Y1s: piece 4pp + 2g + m of the L row
    int foff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) foff[u] = unit_piece_off(ln, 4 * (u >> 1) + 2 * g + (u & 1));
    // activation block: Y1s[b][16 * (c*QK/4 + 4*tq + 2*pp + g) ..], 32 bytes = (kk, j%4) for four j
    const uint16_t* abase = y1s + (size_t)ln * C::Y1_STRIDE + 16 * g;

    f32x16 acc[UPW * K];
#pragma unroll
    for (int t = 0; t < UPW * K; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    auto issue = [&](int n) {
        const int c = n / (TQ64 * NLT), tq = (n / NLT) % TQ64, li = n % NLT;
        const uint16_t* src = Lrow + (size_t)c * C::S * C::Q + tq * 64 + (size_t)((li && second_ok) ? 32 : 0) * C::Q;
        uint16_t* dst = stg + (size_t)(n % RD) * 2048;
#pragma unroll
        for (int bi = 0; bi < 4; ++bi) dma16(src + (size_t)bi * 8 * C::Q + 8 * (pe ^ (bi & 1)), dst + bi * 512);
    };
    u32x4 wraw[2][4];
    u32x4 ablk[2][2][C::NB][2];  // [slot][pp][nb][lo/hi 16 bytes of the block]
    auto read = [&](int n, int slot) {
        const int c = n / (TQ64 * NLT), tq = (n / NLT) % TQ64;
        const uint16_t* wbuf = stg + (size_t)(n % RD) * 2048;
        const uint16_t* ap = abase + 16 * (c * (C::QK / 4) + 4 * tq);
#pragma unroll
        for (int u = 0; u < 4; ++u) wraw[slot][u] = lds128(wbuf + foff[u]);
#pragma unroll
        for (int pp = 0; pp < 2; ++pp)
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb) {
                ablk[slot][pp][nb][0] = lds128(ap + (size_t)nb * 32 * C::Y1_STRIDE + 32 * pp);
                ablk[slot][pp][nb][1] = lds128(ap + (size_t)nb * 32 * C::Y1_STRIDE + 32 * pp + 8);
            }
    };
    wait_vmcnt<0>();  // stores of the previous pass: the ring below counts loads only
    // A ring slot is free as soon as its fragments are in registers, one step before their MFMAs:
    // RD units are in flight or landed at any time (unit n + RD is issued in step n).
#pragma unroll
    for (int d = 0; d < RD; ++d)
        if (d < NU) issue(d);
    wait_vmcnt<((NU < RD ? NU : RD) - 1) * 4>();
    __builtin_amdgcn_sched_barrier(0);
    read(0, 0);
#pragma unroll
    for (int n = 0; n < NU; ++n) {
        __builtin_amdgcn_sched_barrier(0);
        wait_lgkmcnt0();  // the fragments of unit n are in registers: its slot is recycled below
        if (n + RD < NU) issue(n + RD);
        if (n + 1 < NU) {
            // unit n+1 has landed once at most the units issued after it are outstanding
            const int later = (n + RD < NU ? n + RD : NU - 1) - (n + 1);
            wait_vmcnt_units(later);
            __builtin_amdgcn_sched_barrier(0);
            read(n + 1, (n + 1) & 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        const int c = n / (TQ64 * NLT), li = n % NLT;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            // piece dwords (r1a,k0 k1) (r1a,k2 k3) (r1b,k0 k1) (r1b,k2 k3) -> slots (kk, r1a r1b)
            const u32x4& p = wraw[n & 1][u];
            const u32x4 wv = {pick_lo16(p[0], p[2]), pick_hi16(p[0], p[2]), pick_lo16(p[1], p[3]), pick_hi16(p[1], p[3])};
            const bf16x8 wfrag = as_bf16x8(wv);
#pragma unroll
            for (int i = 0; i < UPW; ++i) {
                const int ww = i + (ODD ? 1 : 0);  // work unit relative to the first staged l tile
                if ((ww >> 1) == li) {
                    // dword 2*kk + m of the block holds (j%4 = 2m, 2m+1) for kk: slots (kk, r1a r1b)
                    const u32x4& b0v = ablk[n & 1][u >> 1][ww & 1][0];
                    const u32x4& b1v = ablk[n & 1][u >> 1][ww & 1][1];
                    const int m = u & 1;
                    const u32x4 av = {b0v[m], b0v[2 + m], b1v[m], b1v[2 + m]};
                    acc[i * K + c] = mfma32(as_bf16x8(av), wfrag, acc[i * K + c]);
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
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t row = b0 + (ww & 1) * 32 + 8 * (e / 4) + 4 * g + (e % 4);
            if (row < B) {
                u32x2 v = {pack_bf16x2(acc[i * K + 0][e], acc[i * K + 1][e]), pack_bf16x2(acc[i * K + 2][e], acc[i * K + 3][e])};
                __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(y + row * C::N_OUT + (size_t)l * K));
            }
        }
    }
}

// Stage 2 on 32-column chunks (64 bytes per row).  One pass of one wave: units u0 .. u0+UPW-1,
// unit u = (l tile u / 2, row tile u % 2).
template <typename C, bool ODD>
__device__ __forceinline__ void stage2_pass(const uint16_t* __restrict__ L, const uint16_t* y1s, uint16_t* stg,
                                            uint16_t* __restrict__ y, int64_t b0, int64_t B, int u0, int lane)
{
    constexpr int UPW = C::UPW, K = 4;
    const int ln = lane & 31, g = lane >> 5;
    const int lt_lo = u0 >> 1;
    // staging source: lane s covers row s/4 of a 16-row block, stored piece s%4 holds logical piece p
    const int sr = lane >> 2, sp = (lane & 3) ^ ((sr >> 2) & 3);
    const uint16_t* Lsrc = L + ((size_t)lt_lo * 32 + sr) * C::Q + 8 * sp;
    // fragment read offsets inside a staged 32-row tile (two blocks), K-step u of the chunk
    const int rr = ln & 15, sw = (rr >> 2) & 3;
    // K-step m of a chunk: lane group g contracts over r = 16g + 8m .. +7 of the chunk's 32 (piece 2g + m)
    const int foff0 = (ln >> 4) * 512 + rr * 32 + 8 * ((2 * g + 0) ^ sw);
    const int foff1 = (ln >> 4) * 512 + rr * 32 + 8 * ((2 * g + 1) ^ sw);
    // activation block: Y1s[b][16 * (c*QK/4 + 2*tq + g) ..], 32 bytes = (kk, j%4) for four j
    const uint16_t* abase = y1s + (size_t)ln * C::Y1_STRIDE + 16 * g;

    f32x16 acc[UPW * K];
#pragma unroll
    for (int t = 0; t < UPW * K; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    constexpr int NST = K * C::TQ;
    auto issue = [&](int st) {
        const int c = st / C::TQ, tq = st - c * C::TQ;
        const uint16_t* src = Lsrc + (size_t)c * C::S * C::Q + tq * 32;
        uint16_t* dst = stg + (size_t)(st % C::D2) * C::NBLK2 * 512;
#pragma unroll
        for (int blk = 0; blk < C::NBLK2; ++blk) {
            // the last l tile of the table is only touched by odd-aligned waves; clamp its rows
            int roff = blk * 16;
            if (lt_lo * 32 + roff + 16 > C::S) roff = 0;
            dma16(src + (size_t)roff * C::Q, dst + blk * 512);
        }
    };
    wait_vmcnt<0>();  // stores of the previous pass: the ring below counts loads only
#pragma unroll
    for (int d = 0; d < C::D2 - 1; ++d)
        if (d < NST) issue(d);

#pragma unroll
    for (int c = 0; c < K; ++c) {
        for (int tq = 0; tq < C::TQ; ++tq) {
            const int st = c * C::TQ + tq;
            __builtin_amdgcn_sched_barrier(0);
            if (st + C::D2 - 1 < NST) {
                issue(st + C::D2 - 1);
                wait_vmcnt<(C::D2 - 1) * C::NBLK2>();
            } else if (C::D2 >= 3 && st + C::D2 - 2 < NST) {
                wait_vmcnt<(C::D2 >= 3 ? C::D2 - 2 : 0) * C::NBLK2>();
            } else {
                wait_vmcnt<0>();
            }
            __builtin_amdgcn_sched_barrier(0);
            const uint16_t* wbuf = stg + (size_t)(st % C::D2) * C::NBLK2 * 512;
            const uint16_t* ap = abase + 16 * (c * (C::QK / 4) + 2 * tq);
            u32x4 ablk[C::NB][2];
#pragma unroll
            for (int nb = 0; nb < C::NB; ++nb) {
                ablk[nb][0] = lds128(ap + (size_t)nb * 32 * C::Y1_STRIDE);
                ablk[nb][1] = lds128(ap + (size_t)nb * 32 * C::Y1_STRIDE + 8);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                bf16x8 wfr[C::NLT], afr[C::NB];
#pragma unroll
                for (int li = 0; li < C::NLT; ++li) {
                    const u32x4 p = lds128(wbuf + li * 1024 + (u ? foff1 : foff0));
                    // piece dwords (r1a,k0 k1) (r1a,k2 k3) (r1b,k0 k1) (r1b,k2 k3) -> slots (kk, r1a r1b)
                    const u32x4 wv = {pick_lo16(p[0], p[2]), pick_hi16(p[0], p[2]), pick_lo16(p[1], p[3]), pick_hi16(p[1], p[3])};
                    wfr[li] = as_bf16x8(wv);
                }
#pragma unroll
                for (int nb = 0; nb < C::NB; ++nb) {
                    // dword 2*kk + u of the block holds (j%4 = 2u, 2u+1) for kk: slots (kk, r1a r1b)
                    const u32x4 av = {ablk[nb][0][u], ablk[nb][0][2 + u], ablk[nb][1][u], ablk[nb][1][2 + u]};
                    afr[nb] = as_bf16x8(av);
                }
#pragma unroll
                for (int i = 0; i < UPW; ++i) {
                    const int uu = i + (ODD ? 1 : 0);  // unit index relative to the first staged l tile
                    acc[i * K + c] = mfma32(afr[uu & 1], wfr[uu >> 1], acc[i * K + c]);
                }
            }
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    // step 3: y[b][4*l + c]; lane holds D[b][l] for l = lt*32 + ln, b = nb*32 + 8*(i/4) + 4*g + i%4
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
        const int uu = i + (ODD ? 1 : 0);
        const int l = (lt_lo + (uu >> 1)) * 32 + ln;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t row = b0 + (uu & 1) * 32 + 8 * (e / 4) + 4 * g + (e % 4);
            if (row < B) {
                u32x2 v = {pack_bf16x2(acc[i * K + 0][e], acc[i * K + 1][e]), pack_bf16x2(acc[i * K + 2][e], acc[i * K + 3][e])};
                __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(y + row * C::N_OUT + (size_t)l * K));
            }
        }
    }
}

// SAVE: the vector between the two factors is also written out, in stage-2 order U[b][c*Q + r]
// (r = 4*r1 + kk  <->  Y1[b][kk][c*Q/4 + r1]), for a backward that does not recompute it.
template <typename C, bool SAVE>
__global__ void __launch_bounds__(256)
fwd_wide_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ R,
                const uint16_t* __restrict__ L, uint16_t* __restrict__ y, uint16_t* __restrict__ saved, int64_t B)
{
    extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 31, g = lane >> 5;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;

    // ------------------------------------------------------------- stage 1 ----
    {
        const int kk = wave;
        uint16_t* stg = lds + (size_t)wave * (C::STG1 / 2);
        // The wave consumes a stream of 4 KiB units, per 64-column chunk: x rows 0..31, x rows 32..63,
        // then the R tiles j = 0..31, 32..63, ...  Unit n sits in ring slot n % RD1.
        const int rb = lane >> 3, pe = (lane & 7) ^ rb;
        const uint16_t* Rrow = R + ((size_t)kk * C::Q + rb) * C::P;
        const uint16_t* Xrow[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int64_t row = b0 + i * 8 + rb;
            row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and dropped
            Xrow[i] = x + row * C::N_IN + kk * C::P;
        }
        auto issue = [&](int c64, int u) {  // u static: 0, 1 = x units; 2.. = R tile u - 2
            uint16_t* dst = stg + (size_t)((c64 * C::UPC + u) % C::RD1) * 2048;
#pragma unroll
            for (int bi = 0; bi < 4; ++bi) {
                const uint16_t* src = u < 2 ? Xrow[u * 4 + bi] : Rrow + (size_t)((u - 2) * 32 + bi * 8) * C::P;
                dma16(src + c64 * 64 + 8 * (pe ^ (bi & 1)), dst + bi * 512);
            }
        };
        int foff[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) foff[u] = unit_frag_off(ln, g, u);

        f32x16 acc[C::QT * C::NB];
#pragma unroll
        for (int t = 0; t < C::QT * C::NB; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

        u32x4 xf[C::NB][4], rf[2][4];
        auto read = [&](int c64, int u, u32x4 (&dst)[4]) {
            const uint16_t* buf = stg + (size_t)((c64 * C::UPC + u) % C::RD1) * 2048;
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) dst[k4] = lds128(buf + foff[k4]);
        };
        // prologue: units 0 .. RD1-2 of the stream
#pragma unroll
        for (int d = 0; d < C::RD1 - 1; ++d)
            if (d < C::NU1) issue(d / C::UPC, d % C::UPC);
        wait_vmcnt<((C::NU1 < C::RD1 - 1 ? C::NU1 : C::RD1 - 1) - 1) * 4>();
        __builtin_amdgcn_sched_barrier(0);
        read(0, 0, xf[0]);

        for (int c64 = 0; c64 < C::C1; ++c64) {
#pragma unroll
            for (int u = 0; u < C::UPC; ++u) {
                const int n = c64 * C::UPC + u;
                __builtin_amdgcn_sched_barrier(0);
                wait_lgkmcnt0();  // no fragment read may still be pending on the slot recycled below
                {
                    constexpr int dummy = 0; (void)dummy;
                    const int ui = (u + C::RD1 - 1) % C::UPC, ci = c64 + (u + C::RD1 - 1) / C::UPC;
                    if (n + C::RD1 - 1 < C::NU1) issue(ci, ui);
                }
                const bool next_is_x = (u + 1 == C::UPC) || (u + 1 < 2);
                const int un = (u + 1) % C::UPC, cn = c64 + (u + 1) / C::UPC;
                auto wait_next = [&]() {
                    // unit n+1 has landed once only the units issued after it are outstanding
                    if (n + C::RD1 - 1 < C::NU1) wait_vmcnt<(C::RD1 - 2) * 4>(); else wait_vmcnt<0>();
                    __builtin_amdgcn_sched_barrier(0);
                };
                if (!next_is_x && n + 1 < C::NU1) {
                    wait_next();
                    read(cn, un, rf[un & 1]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (u >= 2) {
                    const int jt = u - 2;
#pragma unroll
                    for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
                        for (int nb = 0; nb < C::NB; ++nb)
                            acc[jt * C::NB + nb] = mfma32(as_bf16x8(rf[u & 1][k4]), as_bf16x8(xf[nb][k4]), acc[jt * C::NB + nb]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (next_is_x && n + 1 < C::NU1) {
                    wait_next();
                    read(cn, un, xf[un]);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();  // every wave is done with its staging ring: the space becomes Y1s
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
        uint16_t* stg = lds + C::LDS_Y1 / 2 + (size_t)wave * (C::STG2 / 2);
        // short batches: gridDim.y workgroups share a row tile, each with a contiguous share of the stage-2 passes
        // (its own columns of y and part of L) after computing stage 1 for itself
        const int ps_lo = (int)blockIdx.y * C::PASSES / (int)gridDim.y, ps_hi = ((int)blockIdx.y + 1) * C::PASSES / (int)gridDim.y;
        for (int ps = ps_lo; ps < ps_hi; ++ps) {
            const int u0 = (ps * 4 + wave) * C::UPW;
            if constexpr (C::S2_LINES) {
                if (u0 & 1)
                    stage2_pass_lines<C, true>(L, lds, stg, y, b0, B, u0, lane);
                else
                    stage2_pass_lines<C, false>(L, lds, stg, y, b0, B, u0, lane);
            } else {
                if (u0 & 1)
                    stage2_pass<C, true>(L, lds, stg, y, b0, B, u0, lane);
                else
                    stage2_pass<C, false>(L, lds, stg, y, b0, B, u0, lane);
            }
        }
    }
    // Last, so that nothing in stage 2 queues behind these stores (Y1s is only read after stage 1).
    if constexpr (SAVE) {
        if (blockIdx.y != 0) return;  // one of the workgroups that share the row tile writes the saved vector
        // Y1s holds, per row and per group of four j, the 16 values [kk][j % 4]; U wants them as [j % 4][kk]
        // (U index 4*j + kk): a 4 x 4 transpose of 16-bit values inside each 32-byte group, then 32
        // contiguous bytes per group and 2*K*Q contiguous bytes per row go out.
        // Two lanes share a group, each writing one 16-byte half, so that a store instruction of a wave
        // covers 1 KiB of contiguous output (full cache lines).
        constexpr int PIECES = C::KQ / 8, TASKS = C::BM * PIECES;
#pragma unroll 4
        for (int t = tid; t < TASKS; t += 256) {
            const int row = t / PIECES, pc = t - row * PIECES;
            const int gq = pc >> 1, half = pc & 1;
            if (b0 + row < B) {
                const uint16_t* src = lds + (size_t)row * C::Y1_STRIDE + gq * 16;
                const u32x4 a = lds128(src), b = lds128(src + 8);
                const uint32_t in[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
                uint32_t o[4];
#pragma unroll
                for (int w4 = 0; w4 < 4; ++w4) {
                    // output dword w = 4*half + w4 holds (j % 4 = w / 2; kk = 2*(w % 2), 2*(w % 2) + 1)
                    const int k0 = 2 * (w4 & 1);
                    const uint32_t lo0 = in[k0 * 2], hi0 = in[(k0 + 1) * 2];          // j % 4 in {0, 1}
                    const uint32_t lo1 = in[k0 * 2 + 1], hi1 = in[(k0 + 1) * 2 + 1];  // j % 4 in {2, 3}
                    const uint32_t lo = half ? lo1 : lo0, hi = half ? hi1 : hi0;
                    o[w4] = (w4 >> 1) ? pick_hi16(lo, hi) : pick_lo16(lo, hi);
                }
                stg128_nt(saved + (b0 + row) * C::KQ + pc * 8, u32x4{o[0], o[1], o[2], o[3]});
            }
        }
    }
}

template <typename C>
int launch(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    auto kern = pb.saved ? fwd_wide_kernel<C, true> : fwd_wide_kernel<C, false>;
    hipError_t e = allow_dynamic_lds((const void*)kern, C::LDS_BYTES);
    if (e != hipSuccess) return -4;
    const int64_t grid = (pb.B + C::BM - 1) / C::BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid, (unsigned)pass_split(grid, C::PASSES)), dim3(256), C::LDS_BYTES, st,
                       (const uint16_t*)x, (const uint16_t*)R, (const uint16_t*)L, (uint16_t*)y, (uint16_t*)pb.saved, pb.B);
    return hip_status(hipGetLastError());
}

struct Entry {
    int p, q, s;
    int (*fn)(const Problem&, const void*, const void*, const void*, void*, hipStream_t);
};

//                                 P     Q     S  UPW
const Entry kTable[] = {
    {192, 192, 192, launch<FwdWide<192, 192, 192, 3>>},    // ViT-B projection 768 -> 768
    {192, 192, 768, launch<FwdWide<192, 192, 768, 4>>},    // GPT-2 small fc1 768 -> 3072
    {256, 256, 1024, launch<FwdWide<256, 256, 1024, 2>>},  // GPT-2 medium fc1 1024 -> 4096
    {1024, 256, 256, launch<FwdWide<1024, 256, 256, 2>>},  // GPT-2 medium fc2 4096 -> 1024
    {768, 192, 192, launch<FwdWide<768, 192, 192, 3>>},    // GPT-2 small fc2 3072 -> 768
    {256, 256, 256, launch<FwdWide<256, 256, 256, 2>>},    // GPT-2 medium projection 1024 -> 1024
    {192, 192, 576, launch<FwdWide<192, 192, 576, 3>>},    // ViT-B / GPT-2 small fused q,k,v 768 -> 2304
    {256, 256, 768, launch<FwdWide<256, 256, 768, 2>>},    // GPT-2 medium fused q,k,v 1024 -> 3072
    {128, 128, 128, launch<FwdWide<128, 128, 128, 2>>},    // width 512 (MLP-Mixer-S): 512 -> 512
    {128, 128, 512, launch<FwdWide<128, 128, 512, 4>>},    // 512 -> 2048
    {512, 128, 128, launch<FwdWide<512, 128, 128, 2>>},    // 2048 -> 512
    {64, 64, 64, launch<FwdWide<64, 64, 64, 1>>},          // small shapes (tests)
    {64, 64, 128, launch<FwdWide<64, 64, 128, 2>>},
    {128, 64, 64, launch<FwdWide<128, 64, 64, 1>>},
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
