// Step 1 of Section 3.3 as a batched GEMM of its own, for the backward pass of the bf16 "wide block"
// layers (k = 4):   Y1[b][kk*Q + j] = sum_i R[kk][j][i] * x[b][kk*P + i]   written to the workspace,
// where the weight-gradient GEMM (dL) reads it.
//
// Why not inside the backward's data kernel (which can also do it, 64 rows per workgroup): there every
// workgroup streams the whole of R through its CU's L1 for 64 rows, and for layers with long blocks
// (p = 1024: R is 2 MB) that stream is the larger half of the kernel.  Y1 has to go through the
// workspace anyway, so nothing ties this product to 64-row tiles: here a workgroup takes 256 rows of
// one block (192 for q = 192), so R passes each L1 a quarter as often.  Used for p >= 768 (see the table below).
//
//   workgroup  = (row tile of BM = 32 * NW rows, block kk); NW = 8 waves (6 for q = 192)
//   x          travels in 64-column chunks through an LDS ring of XR = 4 slots filled by
//              global_load_lds_dwordx4 (each wave fetches 32 rows of every chunk, full 128-byte lines,
//              the swizzled unit layout of monarch_mfma_stage1.h); one barrier per chunk publishes the
//              chunk and frees the slot of the chunk before it
//   R          comes packed in fragment order (the XF array of the backward's prep pass) straight
//              into registers, a chunk (four K-steps) ahead; wave w owns the 32 columns j of tile w % QT
//              (and, when q < 256, the w / QT-th share of the rows), so no fragment is fetched twice
//   D^T        = R . X^T on v_mfma_f32_32x32x16_bf16, at most eight 32 x 32 accumulators per wave
//   Y1         leaves through LDS (the ring's space) in full rows: 16-byte pieces, 2*Q contiguous bytes per row
#include "monarch_internal.h"
#include "monarch_mfma_common.h"
#include "monarch_mfma_stage1.h"
#include <type_traits>

namespace monarch {

namespace {

// (Half as many rows per workgroup, two workgroups per CU so that one's copy-out overlaps the other's streaming:
// measured the same, 46 us for 4096 -> 1024; not kept.)
template <int P_, int Q_>
struct Y1Gemm {
    static constexpr int P = P_, Q = Q_, K = 4;
    static constexpr int QT = Q / 32;                  // 32-wide column tiles of a block
    static constexpr int NW = QT == 6 ? 6 : 8;         // waves
    static constexpr int RSPLIT = NW / QT;             // waves that share a column tile, each with its share of the rows
    static constexpr int BM = 32 * NW;                 // rows per workgroup
    static constexpr int UNITS = BM / 32;              // 32-row DMA units per chunk: one per wave
    static constexpr int DPW = 4;                      // DMA instructions per wave and chunk
    static constexpr int RTW = UNITS / RSPLIT;         // 32-row tiles per wave
    static constexpr int C1 = P / 64, T1 = P / 16;
    static constexpr int XR = 4, D = XR - 1;           // ring slots; chunks requested ahead
    static constexpr int SLOT = BM * 64;               // elements per slot (BM rows x 128 bytes)
    static constexpr int OUT_STRIDE = Q + 8;
    static constexpr size_t LDS_RING = (size_t)XR * SLOT * 2, LDS_OUT = (size_t)BM * OUT_STRIDE * 2;
    static constexpr size_t LDS_BYTES = LDS_RING > LDS_OUT ? LDS_RING : LDS_OUT;
    static_assert(P % 64 == 0 && Q % 64 == 0 && NW % QT == 0 && C1 >= D, "tile shapes");
    static_assert(RTW * RSPLIT == UNITS && RTW <= 8 && UNITS == NW, "row split");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

template <typename C>
__global__ void __launch_bounds__(C::NW * 64)
y1_gemm_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ XF, uint16_t* __restrict__ Y1, int64_t B)
{
    extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int ln = lane & 31, g = lane >> 5;
    const int kk = blockIdx.y;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;
    const int jt = wave % C::QT, rs = wave / C::QT;

    // this wave's 32 rows of every x chunk: four DMA instructions, lane s <- row s/8, piece (s%8) ^ key
    const int rb = lane >> 3, pe = (lane & 7) ^ rb;
    const uint16_t* Xrow[C::DPW];
#pragma unroll
    for (int i = 0; i < C::DPW; ++i) {
        int64_t row = b0 + wave * 32 + i * 8 + rb;
        row = row < B ? row : B - 1;  // rows past the end are computed from a valid row and never stored
        Xrow[i] = x + row * (C::K * C::P) + kk * C::P;
    }
    // The chunks are taken in an order rotated by the workgroup's index, so that the workgroups, which run in step,
    // do not all read the same 128-byte column of rows that are a power of two apart at the same time (a plain read
    // of such a matrix gains a third from it; this kernel measured the same with and without).
    const int rot = (int)(blockIdx.x % C::C1);
    auto chunk_of = [&](int seq) { const int c = seq + rot; return c < C::C1 ? c : c - C::C1; };
    auto issue_x = [&](int seq) {
        uint16_t* dst = lds + (size_t)(seq % C::XR) * C::SLOT + wave * 2048;
        const int c64 = chunk_of(seq);
#pragma unroll
        for (int i = 0; i < C::DPW; ++i)
            dma16(Xrow[i] + c64 * 64 + 8 * (pe ^ (i & 1)), dst + i * 512);
    };
    int foff[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) foff[u] = unit_frag_off(ln, g, u);
    // packed R: fragment (kk, t, jt) at ((kk*T1 + t)*QT + jt) * 512 elements, + lane * 8
    const uint16_t* Rk = XF + (((size_t)kk * C::T1 * C::QT + jt) * 64 + lane) * 8;

    f32x16 acc[C::RTW];
#pragma unroll
    for (int t = 0; t < C::RTW; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    // Loads return in the order they were requested, so a wave cannot use an R fragment that it asked for after an
    // x chunk until that chunk (which comes all the way from HBM) has landed.  Hence the order: at the top of chunk c
    // the four fragments of chunk c+1 are requested first, then the DMA of x chunk c+D; nothing is requested while
    // the chunk is being multiplied.  rf holds two chunks of fragments.
    u32x4 rf[8];
    // K-step u of chunk number `seq` of the rotated sequence
    auto issue_r = [&](int seq, int u, int slot) { rf[slot] = ldg128(Rk + (size_t)(chunk_of(seq) * 4 + u) * C::QT * 512); };
#pragma unroll
    for (int u = 0; u < 4; ++u) issue_r(0, u, u);
#pragma unroll
    for (int c = 0; c < C::D; ++c) issue_x(c);

    auto chunk = [&](int c64, auto par) {
        constexpr int PAR = decltype(par)::value;
        // x chunk c64 and the fragments of chunk c64 have landed once only what was requested after the fragments
        // is outstanding: the DMA that followed them (chunk 0: the other x chunks of the prologue)
        if (c64 == 0) wait_vmcnt<C::DPW * (C::D - 1)>();
        else if (c64 - 1 + C::D < C::C1) wait_vmcnt<C::DPW>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_sched_barrier(0);
        lds_barrier();  // every wave's rows of chunk c64 are there, and nobody reads chunk c64-1 any more
        if (c64 + 1 < C::C1) {
#pragma unroll
            for (int u = 0; u < 4; ++u) issue_r(c64 + 1, u, (PAR ^ 1) * 4 + u);
        }
        if (c64 + C::D < C::C1) issue_x(c64 + C::D);
        const uint16_t* slot = lds + (size_t)(c64 % C::XR) * C::SLOT + (size_t)rs * C::RTW * 2048;
        // the x fragments of a K-step are read while the MFMAs of the K-step before run
        u32x4 xf[2][C::RTW];
#pragma unroll
        for (int rt = 0; rt < C::RTW; ++rt) xf[0][rt] = lds128(slot + rt * 2048 + foff[0]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            __builtin_amdgcn_sched_barrier(0);
            if (u < 3) {
#pragma unroll
                for (int rt = 0; rt < C::RTW; ++rt) xf[(u + 1) & 1][rt] = lds128(slot + rt * 2048 + foff[u + 1]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rt = 0; rt < C::RTW; ++rt) acc[rt] = mfma32(as_bf16x8(rf[PAR * 4 + u]), as_bf16x8(xf[u & 1][rt]), acc[rt]);
        }
    };
    for (int c64 = 0; c64 < C::C1; c64 += 2) {
        chunk(c64, std::integral_constant<int, 0>{});
        if (c64 + 1 < C::C1) chunk(c64 + 1, std::integral_constant<int, 1>{});
    }
    __builtin_amdgcn_sched_barrier(0);
    lds_barrier();  // the ring is no longer read: its space becomes the output tile [BM][OUT_STRIDE]
    // lane holds D^T[j][b] for b = (rs*RTW + rt)*32 + ln and j = jt*32 + 8*(i/4) + 4*g + i%4
#pragma unroll
    for (int rt = 0; rt < C::RTW; ++rt)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const f32x16& a = acc[rt];
            const int j = jt * 32 + 8 * i4 + 4 * g;
            *reinterpret_cast<u32x2*>(lds + (size_t)((rs * C::RTW + rt) * 32 + ln) * C::OUT_STRIDE + j) =
                u32x2{pack_bf16x2(a[4 * i4 + 0], a[4 * i4 + 1]), pack_bf16x2(a[4 * i4 + 2], a[4 * i4 + 3])};
        }
    lds_barrier();
    // rows out: 16-byte pieces, consecutive lanes along a row (the weight-gradient GEMM reads them next: cached stores)
    constexpr int PER_ROW = C::Q / 8, TASKS = C::BM * PER_ROW, NTHR = C::NW * 64;
    static_assert(TASKS % NTHR == 0, "copy-out split");
#pragma unroll 4
    for (int t = tid; t < TASKS; t += NTHR) {
        const int r = t / PER_ROW, u = t % PER_ROW;
        if (b0 + r < B)
            *reinterpret_cast<u32x4*>(Y1 + (b0 + r) * (C::K * C::Q) + kk * C::Q + 8 * u) =
                lds128(lds + (size_t)r * C::OUT_STRIDE + 8 * u);
    }
}

template <typename C>
int launch(const Problem& pb, const void* x, const uint16_t* XF, uint16_t* Y1, hipStream_t st)
{
    auto kern = y1_gemm_kernel<C>;
    if (allow_dynamic_lds((const void*)kern, C::LDS_BYTES) != hipSuccess) return -4;
    const int64_t tiles = (pb.B + C::BM - 1) / C::BM;
    if (tiles > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles, 4), dim3(C::NW * 64), C::LDS_BYTES, st, (const uint16_t*)x, XF, Y1, pb.B);
    return hip_status(hipGetLastError());
}

struct Entry {
    int p, q;
    int (*fn)(const Problem&, const void*, const uint16_t*, uint16_t*, hipStream_t);
};

// Only the layers with long blocks gain (measured, data kernel + this kernel against the data kernel that recomputes
// step 1 itself: 4096 -> 1024: 59 + 46 us against 112; 1024 -> 4096: 69 + 20 against 88; 768 -> 768: 19 + 17 against 29:
// for short blocks the extra launch, and the copy-out that nothing overlaps, cost more than the R stream saved).
const Entry kTable[] = {
    {768, 192, launch<Y1Gemm<768, 192>>},    // GPT-2 small fc2 3072 -> 768
    {1024, 256, launch<Y1Gemm<1024, 256>>},  // GPT-2 medium fc2 4096 -> 1024
};

const Entry* find(const Problem& pb)
{
    if (pb.dtype != 1 || pb.k != 4 || pb.perm_b()) return nullptr;
    for (const Entry& e : kTable)
        if (e.p == pb.p && e.q == pb.q) return &e;
    return nullptr;
}

}  // namespace

bool y1_gemm_supported(const Problem& pb) { return find(pb) != nullptr; }

int y1_gemm(const Problem& pb, const void* x, const uint16_t* XF, uint16_t* Y1, hipStream_t st)
{
    const Entry* e = find(pb);
    return e ? e->fn(pb, x, XF, Y1, st) : -2;
}

}  // namespace monarch
