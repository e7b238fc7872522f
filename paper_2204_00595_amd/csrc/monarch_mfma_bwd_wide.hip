// bf16 backward for "wide block" Monarch layers (k = 4): the adjoints of steps 3, 2, P^T, 1 of
// Section 3.3 (the paper leaves them to automatic differentiation, Section 4).
//
//   prep      re-lays the weights once per call so that every MFMA operand below is one
//             16-byte load:  LTp[c][kk*Q/4 + r1][l] = L[c][l][4*r1 + kk]   (L transposed, rows in the
//             order the mid permutation scatters them),  RTp[kk][i][.] = R[kk][.][i] (R transposed,
//             columns in the order the chained accumulators of `data` hold them).
//   data      one workgroup per 64 batch rows, wave w <-> R block kk = w:
//               X) recompute step 1, Y1[b][kk][j], and write it to the workspace (dL needs U);
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

namespace monarch {

namespace {

// ------------------------------------------------------------------------ prep ----

// Both re-layouts in one launch, 32 x 32 tiles through LDS; blocks [0, tilesL) do L, the rest R.
//   LTp[c][kk*QK + r1][l] = L[c][l][4*r1 + kk]
//   RTp[kk][i][32*u + 8*h + e] = R[kk][j][i],  j = 32*u + 16*(e/4) + 4*h + e%4   (h = 0..3, e = 0..7)
__global__ void __launch_bounds__(256)
prep_kernel(const uint16_t* __restrict__ L, const uint16_t* __restrict__ R, uint16_t* __restrict__ LTp,
            uint16_t* __restrict__ RTp, int P, int Q, int S)
{
    __shared__ uint16_t tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int tilesL = 4 * (S / 32) * (Q / 32);
    int t = blockIdx.x;
    if (t < tilesL) {
        const int nr = Q / 32, nl = S / 32;
        const int r0 = (t % nr) * 32, l0 = (t / nr % nl) * 32, c = t / (nr * nl);
        const int QK = Q / 4;
        for (int yy = ty; yy < 32; yy += 8) tile[yy][tx] = L[((size_t)c * S + l0 + yy) * Q + r0 + tx];
        __syncthreads();
        for (int yy = ty; yy < 32; yy += 8) {
            const int r = r0 + yy;
            const int kappa = (r & 3) * QK + (r >> 2);
            LTp[((size_t)c * Q + kappa) * S + l0 + tx] = tile[tx][yy];
        }
    } else {
        t -= tilesL;
        const int ni = P / 32, nj = Q / 32;
        const int i0 = (t % ni) * 32, j0 = (t / ni % nj) * 32, kk = t / (ni * nj);
        for (int yy = ty; yy < 32; yy += 8) tile[yy][tx] = R[((size_t)kk * Q + j0 + yy) * P + i0 + tx];
        __syncthreads();
        // thread tx writes destination column j0 + tx of row i0 + yy
        const int h = (tx >> 3) & 3, e = tx & 7;
        const int jsrc = 16 * (e >> 2) + 4 * h + (e & 3);
        for (int yy = ty; yy < 32; yy += 8)
            RTp[((size_t)kk * P + i0 + yy) * Q + j0 + tx] = tile[jsrc][yy];
    }
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
    static constexpr size_t LDS_BYTES = LDS_Y1 > LDS_DW ? (LDS_Y1 > LDS_DX ? LDS_Y1 : LDS_DX) : (LDS_DW > LDS_DX ? LDS_DW : LDS_DX);
    static_assert(P % 16 == 0 && Q % 32 == 0 && S % 32 == 0 && QK % 16 == 0, "tile shapes");
    static_assert(QT % JG == 0 && S % LC == 0 && LC % 32 == 0 && (P / 16) % IG == 0, "loop splits");
    static_assert(DX_COLS % 8 == 0 && (64 % (DX_COLS / 8) == 0), "dx staging copy-out");
    static_assert(LDS_BYTES <= kMaxLdsBytes, "LDS");
};

// cooperative copy of a [64][cols] bf16 LDS tile (row stride `stride`) to global rows b0.. (row pitch ld)
__device__ __forceinline__ void copy_out_tile(const uint16_t* src, int stride, uint16_t* dst, int64_t ld,
                                              int cols, int64_t b0, int64_t B, int tid, int nthreads)
{
    const int per_row = cols / 8;
    for (int t = tid; t < 64 * per_row; t += nthreads) {
        const int r = t / per_row, u = t - r * per_row;
        if (b0 + r < B)
            *reinterpret_cast<u32x4*>(dst + (b0 + r) * ld + 8 * u) = lds128(src + (size_t)r * stride + 8 * u);
    }
}

template <typename C>
__global__ void __launch_bounds__(256)
bwd_wide_data_kernel(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ x,
                     const uint16_t* __restrict__ R, const uint16_t* __restrict__ LTp,
                     const uint16_t* __restrict__ RTp, uint16_t* __restrict__ dx,
                     uint16_t* __restrict__ Y1ws, uint16_t* __restrict__ dY1ws, int64_t B)
{
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int64_t b0 = (int64_t)blockIdx.x * C::BM;
    const int kk = wave;

    // ------------------------------------------------- X: recompute step 1 -> workspace ----
    {
        const int ln = lane & 31, g = lane >> 5;
        const uint16_t* xrow[C::NB];
#pragma unroll
        for (int nb = 0; nb < C::NB; ++nb) {
            int64_t row = b0 + nb * 32 + ln;
            row = row < B ? row : B - 1;
            xrow[nb] = x + row * C::N_IN + kk * C::P + 8 * g;
        }
        const uint16_t* Rk = R + ((size_t)kk * C::Q + ln) * C::P + 8 * g;
        constexpr int T = C::P / 16;
        for (int jg = 0; jg < C::QT / C::JG; ++jg) {
            f32x16 acc[C::JG * C::NB];
#pragma unroll
            for (int t = 0; t < C::JG * C::NB; ++t)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
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
#pragma unroll
            for (int jj = 0; jj < C::JG; ++jj)
#pragma unroll
                for (int nb = 0; nb < C::NB; ++nb)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const f32x16& a = acc[jj * C::NB + nb];
                        u32x2 v = {pack_bf16x2(a[4 * i4 + 0], a[4 * i4 + 1]), pack_bf16x2(a[4 * i4 + 2], a[4 * i4 + 3])};
                        const int j = (jg * C::JG + jj) * 32 + 8 * i4 + 4 * g;
                        *reinterpret_cast<u32x2*>(lds + (size_t)(nb * 32 + ln) * C::Y1_STRIDE + kk * C::Q + j) = v;
                    }
        }
        __syncthreads();
        copy_out_tile(lds, C::Y1_STRIDE, Y1ws, C::KQ, C::KQ, b0, B, tid, 256);
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
        // de-interleave dy[b][4*l + c] into LDS dWs[c][b][l - l0]
        constexpr int RUNS = C::LC / 8;  // 64-byte runs per row
        for (int t0 = 0; t0 < 64 * RUNS; t0 += 256) {
            const int t = t0 + tid;
            const int r = t / RUNS, u = t - r * RUNS;
            int64_t row = b0 + r;
            row = row < B ? row : B - 1;
            const uint16_t* p = dy + row * C::N_OUT + (size_t)(l0 + 8 * u) * 4;
            u32x4 raw[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) raw[w] = ldg128(p + 8 * w);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                u32x4 v;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t lo = raw[w][c >> 1], hi = raw[w][2 + (c >> 1)];
                    v[w] = (c & 1) ? pick_hi16(lo, hi) : pick_lo16(lo, hi);
                }
                *reinterpret_cast<u32x4*>(lds + ((size_t)c * 64 + r) * C::DW_STRIDE + 8 * u) = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < C::K; ++c) {
            // A operand rows: LTp[c][kk*QK + jt*16 + l16][l],  B operand: dWs[c][bt*16 + l16][l]
            const uint16_t* Lc = LTp + ((size_t)c * C::Q + kk * C::QK + l16) * C::S + l0 + 8 * h;
            const uint16_t* Wc = lds + ((size_t)c * 64 + l16) * C::DW_STRIDE + 8 * h;
            constexpr int T = C::LC / 32;
            u32x4 af[2][C::JT];
#pragma unroll
            for (int jt = 0; jt < C::JT; ++jt) af[0][jt] = ldg128(Lc + (size_t)jt * 16 * C::S);
#pragma unroll 2
            for (int t = 0; t < T; ++t) {
                const int cur = t & 1, nxt = cur ^ 1;
                if (t + 1 < T) {
#pragma unroll
                    for (int jt = 0; jt < C::JT; ++jt) af[nxt][jt] = ldg128(Lc + (size_t)jt * 16 * C::S + (t + 1) * 32);
                }
                bf16x8 bfr[C::NBT];
#pragma unroll
                for (int bt = 0; bt < C::NBT; ++bt)
                    bfr[bt] = as_bf16x8(lds128(Wc + (size_t)bt * 16 * C::DW_STRIDE + t * 32));
#pragma unroll
                for (int jt = 0; jt < C::JT; ++jt)
#pragma unroll
                    for (int bt = 0; bt < C::NBT; ++bt)
                        accA[(c * C::JT + jt) * C::NBT + bt] =
                            mfma16(as_bf16x8(af[cur][jt]), bfr[bt], accA[(c * C::JT + jt) * C::NBT + bt]);
            }
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
#pragma unroll
    for (int J = 0; J < C::K * C::JT; ++J)
#pragma unroll
        for (int bt = 0; bt < C::NBT; ++bt)
            *reinterpret_cast<u32x2*>(lds + (size_t)(bt * 16 + l16) * C::Y1_STRIDE + kk * C::Q + J * 16 + 4 * h) = dfr[J][bt];
    __syncthreads();
    copy_out_tile(lds, C::Y1_STRIDE, dY1ws, C::KQ, C::KQ, b0, B, tid, 256);
    __syncthreads();

    // ------------------------------------------------- B: dx from the chained fragments ----
    // K-step u covers j in [32u, 32u+32): lane slots 0..3 <- tile 2u, slots 4..7 <- tile 2u+1;
    // RTp rows are laid out in exactly that order, so its operand is one 16-byte load.
    uint16_t* stage = lds + (size_t)wave * 64 * C::DX_STRIDE;
    const uint16_t* Rt = RTp + ((size_t)kk * C::P + l16) * C::Q + 8 * h;
    constexpr int U = C::Q / 32;
    for (int ig = 0; ig < (C::P / 16) / C::IG; ++ig) {
        f32x4 acc[C::IG * C::NBT];
#pragma unroll
        for (int t = 0; t < C::IG * C::NBT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
        const uint16_t* Rg = Rt + (size_t)ig * C::IG * 16 * C::Q;
        u32x4 af[2][C::IG];
#pragma unroll
        for (int it = 0; it < C::IG; ++it) af[0][it] = ldg128(Rg + (size_t)it * 16 * C::Q);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int cur = u & 1, nxt = cur ^ 1;
            if (u + 1 < U) {
#pragma unroll
                for (int it = 0; it < C::IG; ++it) af[nxt][it] = ldg128(Rg + (size_t)it * 16 * C::Q + (u + 1) * 32);
            }
#pragma unroll
            for (int bt = 0; bt < C::NBT; ++bt) {
                const u32x4 bv = {dfr[2 * u][bt][0], dfr[2 * u][bt][1], dfr[2 * u + 1][bt][0], dfr[2 * u + 1][bt][1]};
                const bf16x8 bfr = as_bf16x8(bv);
#pragma unroll
                for (int it = 0; it < C::IG; ++it)
                    acc[it * C::NBT + bt] = mfma16(as_bf16x8(af[cur][it]), bfr, acc[it * C::NBT + bt]);
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
        __syncthreads();
        copy_out_tile(stage, C::DX_STRIDE, dx + kk * C::P + ig * C::DX_COLS, C::N_IN, C::DX_COLS, b0, B, lane, 64);
        __syncthreads();
    }
}

template <typename C>
int launch_data(const Problem& pb, const void* dy, const void* x, const void* R, const uint16_t* LTp,
                const uint16_t* RTp, void* dx, uint16_t* Y1ws, uint16_t* dY1ws, hipStream_t st)
{
    auto kern = bwd_wide_data_kernel<C>;
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES) != hipSuccess)
        return -4;
    const int64_t grid = (pb.B + C::BM - 1) / C::BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), C::LDS_BYTES, st, (const uint16_t*)dy,
                       (const uint16_t*)x, (const uint16_t*)R, LTp, RTp, (uint16_t*)dx, Y1ws, dY1ws, pb.B);
    return hip_status(hipGetLastError());
}

struct Entry {
    int p, q, s;
    int (*fn)(const Problem&, const void*, const void*, const void*, const uint16_t*, const uint16_t*, void*,
              uint16_t*, uint16_t*, hipStream_t);
};

//                                 P     Q     S   JG   LC  IG
const Entry kTable[] = {
    {192, 192, 192, launch_data<BwdWide<192, 192, 192, 6, 192, 4>>},
    {192, 192, 768, launch_data<BwdWide<192, 192, 768, 6, 256, 4>>},
    {256, 256, 1024, launch_data<BwdWide<256, 256, 1024, 4, 256, 4>>},
    {1024, 256, 256, launch_data<BwdWide<1024, 256, 256, 4, 256, 4>>},
    {768, 192, 192, launch_data<BwdWide<768, 192, 192, 6, 192, 4>>},
    {64, 64, 64, launch_data<BwdWide<64, 64, 64, 2, 64, 4>>},
    {64, 64, 128, launch_data<BwdWide<64, 64, 128, 2, 64, 4>>},
    {128, 64, 64, launch_data<BwdWide<128, 64, 64, 2, 64, 4>>},
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
    size_t off_y1, off_dy1, off_ltp, off_rtp, off_partL, off_partR, total;
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
    int64_t z = (256 + tiles - 1) / tiles;
    const int64_t maxz = (pb.B + 255) / 256;
    if (z > maxz) z = maxz;
    if (z < 1) z = 1;
    const int64_t rpc = ((pb.B + z - 1) / z + 31) / 32 * 32;
    pl.rows_per_chunk = (int)(rpc > 0 ? rpc : 32);
    pl.nz = (int)((pb.B + pl.rows_per_chunk - 1) / pl.rows_per_chunk);
    if (pl.nz < 1) pl.nz = 1;
    size_t off = 0;
    const size_t act = align_up((size_t)(pb.B > 0 ? pb.B : 1) * pb.kq() * 2, 256);
    pl.off_y1 = off;  off += act;
    pl.off_dy1 = off; off += act;
    pl.off_ltp = off; off += align_up(pb.n_L() * 2, 256);
    pl.off_rtp = off; off += align_up(pb.n_R() * 2, 256);
    pl.off_partL = off; off += align_up((size_t)pl.nz * pb.n_L() * 4, 256);
    pl.off_partR = off; off += align_up((size_t)pl.nz * pb.n_R() * 4, 256);
    pl.total = off;
    return pl;
}

}  // namespace

bool bwd_wide_supported(const Problem& pb) { return find(pb) != nullptr && make_plan(pb).ok; }

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
    uint16_t* LTp = (uint16_t*)(w + pl.off_ltp);
    uint16_t* RTp = (uint16_t*)(w + pl.off_rtp);
    const bool f32out = pb.wgrad_f32();
    if (pb.B == 0) {
        int rc = f32out ? launch_fill_zero_f32((float*)dR, pb.n_R(), st) : launch_fill_zero_u16((uint16_t*)dR, pb.n_R(), st);
        if (rc) return rc;
        return f32out ? launch_fill_zero_f32((float*)dL, pb.n_L(), st) : launch_fill_zero_u16((uint16_t*)dL, pb.n_L(), st);
    }
    const int prep_blocks = 4 * (pb.s / 32) * (pb.q / 32) + 4 * (pb.q / 32) * (pb.p / 32);
    hipLaunchKernelGGL(prep_kernel, dim3(prep_blocks), dim3(256), 0, st, (const uint16_t*)L, (const uint16_t*)R,
                       LTp, RTp, pb.p, pb.q, pb.s);
    if (hipGetLastError() != hipSuccess) return -4;
    int rc = e->fn(pb, dy, x, R, LTp, RTp, dx, Y1ws, dY1ws, st);
    if (rc) return rc;

    WgradDesc dl, dr;
    fill_descs(pb, dl, dr);
    dl.A = (const uint16_t*)dy; dl.Bm = Y1ws; dl.P = (float*)(w + pl.off_partL); dl.out = dL;
    dr.A = dY1ws; dr.Bm = (const uint16_t*)x; dr.P = (float*)(w + pl.off_partR); dr.out = dR;
    dl.rows_per_chunk = dr.rows_per_chunk = pl.rows_per_chunk;
    rc = wgrad_gemm_pair(dl, dr, pl.nz, st);
    if (rc) return rc;
    return wgrad_reduce_pair(dl, dr, f32out, pl.nz, st);
}

}  // namespace monarch
