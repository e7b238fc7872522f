// Complex-valued Monarch multiply on the matrix cores (complex64, fp32 arithmetic), for square blocks
// p = q = s in {16, 32, 64} and any k.  The paper's results hold over C (Notation Review); the steps are
// those of Section 3.3 with the permutations of Definition 3.1, the gradients those of monarch_complex.hip.
//
// A complex product is a real product of twice the size: with a vector stored as interleaved (re, im) pairs,
// y = W x over C is  y' = W' x'  over R, where W'[2j+e][2i+t] = (Wr, -Wi; Wi, Wr)[e][t].  The activations are
// therefore used exactly as they lie in memory, and the weights are expanded as they are loaded.
//
// One block-diagonal factor is one launch ("stage"), and the vector between the two factors goes through a
// workspace: at n = 4096 a row of it takes 32 KiB, so a 32-row tile does not fit LDS next to anything else.  A
// workgroup owns one block g and a share of the row tiles: its wave w keeps the expanded weights of 16 outputs
// (32 real rows, the M extent of v_mfma_f32_32x32x2_f32) in registers for the whole launch and streams 32-row
// activation tiles (the N extent) past them; a K = 2 step contracts one component of two complex inputs.
//   D (32 x 32): acc[r] = D[8*(r/4) + 4*(lane/32) + r%4][lane%32]: a lane holds whole complex outputs of one row.
//
// The permutation between the factors is an 8-byte transposition, so it is done where the pieces can be made
// long: the workspace holds the intermediate in tiles  T[row tile][block][index in block][32 rows]  (the
// producer writes, per output index, the 32 rows of its tile as one 256-byte run into the block the consumer
// will read; the consumer's tile is then one contiguous block).  Only the outer permutation (y[b][l*k + c], and
// dy read the same way) moves 8-byte pieces; the workgroups of one row range run on one XCD so that these meet in
// one L2.
//
// Weight gradients: dL[c] = dW[c]^T conj(U[c]),  dR[kk] = dY1[kk]^T conj(x[kk]),  contracted over the batch by the
// same MFMA (K = two rows x one component); a workgroup owns one block and a share of the row tiles, the shares'
// partial results go to the workspace and are summed in a fixed order (no atomics).
//
// Real fp32 layers with square blocks of 32 or 64 run on the same kernels (template flag REAL): a float2 is then two
// consecutive values of a row, the activation side is unchanged, the weights are taken as stored and the
// permutations move single values (see cstage_kernel).
#include "monarch_internal.h"
#include "monarch_device.h"
#include "monarch_mfma_common.h"

namespace monarch {
namespace {

constexpr int kRT = 32;  // batch rows per tile

__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

enum : int { kInNat = 0, kInGather = 1, kInT = 2 };
enum : int { kOutTFwd = 0, kOutTBwd = 1, kOutNat = 2, kOutScatter = 3 };

// stage-1 output f = kk*q + j that lands at position g of the permuted vector (inverse of mid_dest)
__device__ __forceinline__ int mid_src(int g, int k, int q, bool perm_b)
{
    if (!perm_b) { const int j = g / k, kk = g - j * k; return kk * q + j; }
    const int c = g / q, r = g - c * q;
    return r * k + c;
}

__device__ __forceinline__ void lds_store_c2(float2* dst, u32x4 v)  // two complex values to an 8-byte aligned place
{
    dst[0] = make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
    dst[1] = make_float2(__uint_as_float(v.z), __uint_as_float(v.w));
}

// A 32-row tile of one block's complex values, P per row, fetched into registers and later written to LDS.
//   kInNat:    src[row][g*P + i]                          LDS [row][P + 1]
//   kInGather: src[row][i*k + g]                          LDS [row][P + 1]
//   kInT:      src tile (rt, g): [i][32 rows], contiguous LDS [i][32]
// Rows past the end of the batch read as zeros (kInT: the producer wrote zeros there).
// REAL (real fp32 data, two consecutive values per float2): only the gathering form differs, whose pieces are then
// single floats, src[row][i'*k + g] for the 2P real indices i' of the block.
template <int P, int NTHR, int IN, bool REAL = false>
struct ActTile {
    static constexpr int kPieces = (IN == kInGather) ? kRT * P / NTHR : kRT * P / 2 / NTHR;  // per thread
    static constexpr int kStride = (IN == kInT) ? kRT : P + 1;
    static constexpr int kLen = (IN == kInT) ? P * kRT : kRT * (P + 1);
    static_assert((IN == kInGather ? kRT * P : kRT * P / 2) % NTHR == 0, "tile does not divide over the threads");
    u32x4 v[IN == kInGather ? (kPieces + 1) / 2 : kPieces];

    __device__ __forceinline__ void fetch(const float2* __restrict__ src, int64_t rt, int g, int k, int64_t ld, int64_t B, int tid)
    {
        const int64_t row0 = rt * kRT;
        if constexpr (IN == kInNat) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / (P / 2), c2 = idx - row * (P / 2);
                v[n] = (row0 + row < B) ? ldg128(src + (row0 + row) * ld + (size_t)g * P + 2 * c2) : u32x4{0, 0, 0, 0};
            }
        } else if constexpr (IN == kInGather && REAL) {
            const float* srcf = reinterpret_cast<const float*>(src);
#pragma unroll
            for (int n = 0; n < 2 * kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / (2 * P), i = idx - row * (2 * P);
                float t = 0.f;
                if (row0 + row < B) t = srcf[(row0 + row) * (2 * ld) + (size_t)i * k + g];
                v[n / 4][n % 4] = __float_as_uint(t);
            }
        } else if constexpr (IN == kInGather) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / P, i = idx - row * P;
                float2 t = make_float2(0.f, 0.f);
                if (row0 + row < B) t = src[(row0 + row) * ld + (size_t)i * k + g];
                if (n & 1) { v[n / 2].z = __float_as_uint(t.x); v[n / 2].w = __float_as_uint(t.y); }
                else { v[n / 2].x = __float_as_uint(t.x); v[n / 2].y = __float_as_uint(t.y); }
            }
        } else {
            const float2* tile = src + ((size_t)rt * k + g) * (P * kRT);
#pragma unroll
            for (int n = 0; n < kPieces; ++n) v[n] = ldg128(tile + 2 * (tid + n * NTHR));
        }
    }

    __device__ __forceinline__ void to_lds(float2* act, int tid) const
    {
        if constexpr (IN == kInNat) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / (P / 2), c2 = idx - row * (P / 2);
                lds_store_c2(act + row * kStride + 2 * c2, v[n]);
            }
        } else if constexpr (IN == kInGather && REAL) {
            float* actf = reinterpret_cast<float*>(act);
#pragma unroll
            for (int n = 0; n < 2 * kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / (2 * P), i = idx - row * (2 * P);
                actf[row * (2 * kStride) + i] = __uint_as_float(v[n / 4][n % 4]);
            }
        } else if constexpr (IN == kInGather) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / P, i = idx - row * P;
                const u32x4 w = v[n / 2];
                act[row * kStride + i] = (n & 1) ? make_float2(__uint_as_float(w.z), __uint_as_float(w.w))
                                                 : make_float2(__uint_as_float(w.x), __uint_as_float(w.y));
            }
        } else {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) *reinterpret_cast<u32x4*>(act + 2 * (tid + n * NTHR)) = v[n];
        }
    }

    // element i of row `row`
    static __device__ __forceinline__ float2 at(const float2* act, int i, int row)
    {
        return (IN == kInT) ? act[i * kRT + row] : act[row * kStride + i];
    }
};

// out[b][block g][n] = sum_m in[b][block g][m] * Wop[g][n][m],  n < Q, m < P;
// Wop[n][m] = W[g][n][m] (W stored [g][Q][P]) or, CONJT, conj(W[g][m][n]) (W stored [g][P][Q]).
//   kOutTFwd:    element (g, n) is stage-1 output f = g*Q + n; it goes to block c, index r of the permuted vector
//   kOutTBwd:    element (g, n) is position g*Q + n of the permuted vector; it goes to block kk, index j of stage 1
//   kOutNat:     out[row][g*Q + n]
//   kOutScatter: out[row][n*k + g]
// Grid: k * nsplit workgroups of Q/16 waves; workgroup (g, split) takes the row tiles split, split + nsplit, ...
// (split = blockIdx % nsplit with nsplit a multiple of 8 keeps the blocks of one row range on one XCD).
// REAL: real fp32 data and weights, block sizes 2P -> 2Q.  A float2 is then two consecutive values of a row, which
// is what one pair of K = 2 steps contracts, so the activation side is unchanged; the weights are used as they are
// (CONJT: transposed), and since the permutations move single values, the two values of a result pair go to their
// places separately (in the tiled workspace, to the pair slot [index / 2][row][index % 2] of the consumer's block).
template <int P, int Q, int IN, int OUT, bool CONJT, bool REAL = false>
__global__ void __launch_bounds__(4 * Q)
cstage_kernel(const float2* __restrict__ in, const float2* __restrict__ W, float2* __restrict__ out, int64_t B,
              int k, int nsplit, int perm_b)
{
    constexpr int NTHR = 4 * Q;
    using Tile = ActTile<P, NTHR, IN, REAL>;
    constexpr int OSTR = Q + 1;
    __shared__ __align__(16) float2 act[2][Tile::kLen];
    __shared__ __align__(16) float2 ost[OUT == kOutNat ? kRT * OSTR : 1];

    const int g = (int)blockIdx.x / nsplit, split = (int)blockIdx.x - g * nsplit;
    const int tid = threadIdx.x, lane = tid & 63, mt = tid >> 6;
    const int col = lane & 31, kh = lane >> 5, e = lane & 1;
    const int64_t ntiles = (B + kRT - 1) / kRT;
    const int64_t ld_in = (int64_t)k * P, ld_out = (int64_t)k * Q;
    const bool pb = perm_b != 0;

    // this lane's rows of the expanded weights: real row 2*jw + e, for the inputs i = 2u + kh
    float A0[P / 2], A1[P / 2];
    {
        if constexpr (REAL) {
            const int nw = 32 * mt + col;  // this lane's output of the block
            const float* Wf = reinterpret_cast<const float*>(W) + (size_t)g * (4 * P * Q);
#pragma unroll
            for (int u = 0; u < P / 2; ++u) {
                const int i = 2 * u + kh;  // inputs 2i and 2i + 1
                if constexpr (CONJT) {
                    A0[u] = Wf[(size_t)(2 * i) * (2 * Q) + nw];
                    A1[u] = Wf[(size_t)(2 * i + 1) * (2 * Q) + nw];
                } else {
                    const float2 w = *reinterpret_cast<const float2*>(Wf + (size_t)nw * (2 * P) + 2 * i);
                    A0[u] = w.x;
                    A1[u] = w.y;
                }
            }
        } else {
            const int jw = 16 * mt + (col >> 1);
            const float2* Wg = W + (size_t)g * P * Q;
            constexpr float sgn = CONJT ? -1.f : 1.f;
#pragma unroll
            for (int u = 0; u < P / 2; ++u) {
                const int i = 2 * u + kh;
                const float2 w = CONJT ? Wg[i * Q + jw] : Wg[jw * P + i];
                A0[u] = e ? sgn * w.y : w.x;
                A1[u] = e ? w.x : -sgn * w.y;
            }
        }
    }

    Tile pre;
    int64_t rt = split;
    if (rt < ntiles) pre.fetch(in, rt, g, k, ld_in, B, tid);
    for (int it = 0; rt < ntiles; rt += nsplit, ++it) {
        float2* a = act[it & 1];
        pre.to_lds(a, tid);
        lds_barrier();
        if (rt + nsplit < ntiles) pre.fetch(in, rt + nsplit, g, k, ld_in, B, tid);

        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
        for (int u = 0; u < P / 2; ++u) {
            const float2 xv = Tile::at(a, 2 * u + kh, col);
            acc = mfma_f32(A0[u], xv.x, acc);
            acc = mfma_f32(A1[u], xv.y, acc);
        }

        const int64_t row = rt * kRT + col;
        if constexpr (OUT == kOutNat) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    ost[col * OSTR + 16 * mt + 4 * q4 + 2 * kh + h] = make_float2(acc[4 * q4 + 2 * h], acc[4 * q4 + 2 * h + 1]);
            lds_barrier();
            constexpr int kPieces = kRT * Q / 2 / NTHR;
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, r = idx / (Q / 2), c2 = idx - r * (Q / 2);
                const float2 v0 = ost[r * OSTR + 2 * c2], v1 = ost[r * OSTR + 2 * c2 + 1];
                if (rt * kRT + r < B)
                    *reinterpret_cast<f32x4*>(out + (rt * kRT + r) * ld_out + (size_t)g * Q + 2 * c2) = f32x4{v0.x, v0.y, v1.x, v1.y};
            }
        } else {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int j = 16 * mt + 4 * q4 + 2 * kh + h;
                    const float2 v = make_float2(acc[4 * q4 + 2 * h], acc[4 * q4 + 2 * h + 1]);
                    if constexpr (REAL) {
                        float* outf = reinterpret_cast<float*>(out);
#pragma unroll
                        for (int t = 0; t < 2; ++t) {
                            const int n = 2 * j + t;  // output of the block, 0 .. 2Q-1
                            const float val = t ? v.y : v.x;
                            if constexpr (OUT == kOutScatter) {
                                if (row < B) outf[row * (2 * ld_out) + (size_t)n * k + g] = val;
                            } else {
                                const int d = (OUT == kOutTFwd) ? mid_dest(g * 2 * Q + n, k, 2 * Q, pb) : mid_src(g * 2 * Q + n, k, 2 * Q, pb);
                                const int blk = d / (2 * Q), idx = d - blk * (2 * Q);
                                outf[((((size_t)rt * k + blk) * Q + (idx >> 1)) * kRT + col) * 2 + (idx & 1)] = val;
                            }
                        }
                    } else if constexpr (OUT == kOutScatter) {
                        if (row < B) out[row * ld_out + (size_t)j * k + g] = v;
                    } else {
                        const int d = (OUT == kOutTFwd) ? mid_dest(g * Q + j, k, Q, pb) : mid_src(g * Q + j, k, Q, pb);
                        const int blk = d / Q, idx = d - blk * Q;
                        out[(((size_t)rt * k + blk) * Q + idx) * kRT + col] = v;
                    }
                }
        }
    }
}

// The two stages that touch the outer permutation (y[b][l*k + c] written, dy read the same way), for k a multiple
// of 8: eight blocks per workgroup, wave w = block 8*oct + w, every wave the same MTW M tiles (16 outputs each) of its
// own block, so that the pieces of the permuted side are the eight blocks' values of one (row, l): 64 contiguous bytes
// instead of 8.  Workgroups that differ only in their M tiles read the same activations (they sit on one XCD); where
// that re-reading costs more than the lost occupancy a wave takes two M tiles (measured: the scattering stage at blocks
// of 64, four M tiles; the gathering stage at blocks of 32).
//
// cscatter8_kernel: tiled workspace -> y.  The activations of a wave's block are MFMA operands exactly as they lie
// in the workspace (lane = row, 512 contiguous bytes per wave load), so they go from global memory to registers
// directly, ahead of the MFMAs; the results are exchanged through LDS as [row][l][block].
template <int P>
constexpr int kMTilesPerWave = P >= 64 ? 2 : 1;
// the gathering stage has less room (its chunk staging registers): two M tiles per wave would spill at blocks of 64,
// and only pay at the batch sizes of the real fp32 layers with blocks of 64 (P = 32 pairs)
template <int P, bool REAL>
constexpr int kMTilesPerWaveGather = (REAL && P == 32) ? 2 : 1;

template <int P, int Q>
struct Scatter8 {
    static constexpr int MTW = kMTilesPerWave<Q>;
    static constexpr int kRow = 16 * MTW * 8 + 1;  // values per row of the exchange buffer
    static constexpr size_t kLds = 2 * (size_t)kRT * kRow * sizeof(float2);
};

// REAL (see cstage_kernel): the pieces of y are the eight blocks' values of one (row, output), 32 bytes.
template <int P, int Q, bool REAL = false>
__global__ void __launch_bounds__(512)
cscatter8_kernel(const float2* __restrict__ T, const float2* __restrict__ W, float2* __restrict__ out, int64_t B, int k,
                 int nsplit)
{
    constexpr int MTW = Scatter8<P, Q>::MTW;
    constexpr int MTG = Q / 16 / MTW;  // groups of M tiles = workgroups per (block octet, split)
    constexpr int NCH = MTW == 1 ? 1 : 4;  // pieces a tile's activations are fetched in
    constexpr int CH = P / 2 / NCH;        // input pairs per piece
    constexpr int OROW = Scatter8<P, Q>::kRow;
    extern __shared__ __align__(16) float2 ost8[];

    int bid = (int)blockIdx.x;
    const int split = bid % nsplit;
    bid /= nsplit;
    const int mt0 = (bid % MTG) * MTW, oct = bid / MTG;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g = 8 * oct + w;
    const int col = lane & 31, kh = lane >> 5, e = lane & 1;
    const int64_t ntiles = (B + kRT - 1) / kRT;
    const int64_t ld_out = (int64_t)k * Q;

    float A0[MTW][P / 2], A1[MTW][P / 2];
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
        if constexpr (REAL) {
            const float* Wf = reinterpret_cast<const float*>(W) + (size_t)g * (4 * P * Q) + (size_t)(32 * (mt0 + m) + col) * (2 * P);
#pragma unroll
            for (int u = 0; u < P / 2; ++u) {
                const float2 wv = *reinterpret_cast<const float2*>(Wf + 2 * (2 * u + kh));
                A0[m][u] = wv.x;
                A1[m][u] = wv.y;
            }
        } else {
            const int jw = 16 * (mt0 + m) + (col >> 1);
            const float2* Wg = W + (size_t)g * P * Q;
#pragma unroll
            for (int u = 0; u < P / 2; ++u) {
                const float2 wv = Wg[jw * P + 2 * u + kh];
                A0[m][u] = e ? wv.y : wv.x;
                A1[m][u] = e ? wv.x : -wv.y;
            }
        }
    }
    auto load = [&](float2 (&buf)[CH], int64_t rt, int part) {
        const float2* src = T + ((size_t)rt * k + g) * (P * kRT) + (size_t)(2 * part * CH + kh) * kRT + col;
#pragma unroll
        for (int u = 0; u < CH; ++u) buf[u] = src[2 * u * kRT];
    };
    f32x16 acc[MTW];
    auto zero = [&]() {
#pragma unroll
        for (int m = 0; m < MTW; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][r] = 0.f;
    };
    auto mma = [&](const float2 (&buf)[CH], int part) {
#pragma unroll
        for (int u = 0; u < CH; ++u)
#pragma unroll
            for (int m = 0; m < MTW; ++m) {
                acc[m] = mfma_f32(A0[m][part * CH + u], buf[u].x, acc[m]);
                acc[m] = mfma_f32(A1[m][part * CH + u], buf[u].y, acc[m]);
            }
    };
    // the results of one tile: exchange through LDS buffer it & 1 (one barrier per tile), then the 64-byte (REAL:
    // 32-byte) pieces of y
    auto emit = [&](int64_t rt, int it) {
        float2* o = ost8 + (it & 1) * (kRT * OROW);
        if constexpr (REAL) {
            // [row][32 * MTW outputs][8 blocks] floats in the same space; acc[m][r] is output 8*(r/4) + 4*kh + r%4 of M tile m
            float* of = reinterpret_cast<float*>(o);
#pragma unroll
            for (int m = 0; m < MTW; ++m)
#pragma unroll
                for (int r = 0; r < 16; ++r) of[col * (2 * OROW) + (32 * m + 8 * (r / 4) + 4 * kh + (r % 4)) * 8 + w] = acc[m][r];
            lds_barrier();
            float* outf = reinterpret_cast<float*>(out);
#pragma unroll
            for (int n = 0; n < 4 * MTW; ++n) {  // 32 rows x 32 * MTW outputs x 2 halves of the eight blocks, 16 bytes each
                const int idx = tid + n * 512, part = idx & 1, nl = (idx >> 1) % (32 * MTW), r = idx / (64 * MTW);
                const float2 v0 = *reinterpret_cast<const float2*>(of + r * (2 * OROW) + nl * 8 + 4 * part);
                const float2 v1 = *reinterpret_cast<const float2*>(of + r * (2 * OROW) + nl * 8 + 4 * part + 2);
                if (rt * kRT + r < B)
                    *reinterpret_cast<f32x4*>(outf + (rt * kRT + r) * (2 * ld_out) + (size_t)(32 * mt0 + nl) * k + 8 * oct + 4 * part) =
                        f32x4{v0.x, v0.y, v1.x, v1.y};
            }
        } else {
#pragma unroll
            for (int m = 0; m < MTW; ++m)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        o[col * OROW + (16 * m + 4 * q4 + 2 * kh + h) * 8 + w] = make_float2(acc[m][4 * q4 + 2 * h], acc[m][4 * q4 + 2 * h + 1]);
            lds_barrier();
#pragma unroll
            for (int n = 0; n < 4 * MTW; ++n) {  // 32 rows x 16 * MTW outputs x 4 pairs of blocks, 16 bytes each
                const int idx = tid + n * 512, c2 = idx & 3, ll = (idx >> 2) % (16 * MTW), r = idx / (64 * MTW);
                const float2 v0 = o[r * OROW + ll * 8 + 2 * c2], v1 = o[r * OROW + ll * 8 + 2 * c2 + 1];
                if (rt * kRT + r < B)
                    *reinterpret_cast<f32x4*>(out + (rt * kRT + r) * ld_out + (size_t)(16 * mt0 + ll) * k + 8 * oct + 2 * c2) =
                        f32x4{v0.x, v0.y, v1.x, v1.y};
            }
        }
    };

    // two register sets: the next piece of the activations (a whole tile, or a quarter where the weights of two M
    // tiles leave less room) is on its way while the current one is multiplied
    float2 xa[CH], xb[CH];
    int64_t rt = split;
    if (rt < ntiles) load(xa, rt, 0);
    if constexpr (NCH == 1) {
        for (int it = 0; rt < ntiles; it += 2) {
            if (rt + nsplit < ntiles) load(xb, rt + nsplit, 0);
            zero();
            mma(xa, 0);
            emit(rt, it);
            rt += nsplit;
            if (rt >= ntiles) break;
            if (rt + nsplit < ntiles) load(xa, rt + nsplit, 0);
            zero();
            mma(xb, 0);
            emit(rt, it + 1);
            rt += nsplit;
        }
    } else {
        for (int it = 0; rt < ntiles; rt += nsplit, ++it) {
            zero();
            load(xb, rt, 1);
            mma(xa, 0);
            load(xa, rt, 2);
            mma(xb, 1);
            load(xb, rt, 3);
            mma(xa, 2);
            if (rt + nsplit < ntiles) load(xa, rt + nsplit, 0);
            mma(xb, 3);
            emit(rt, it);
        }
    }
}

// cgather8_kernel: dy (read through the outer permutation) -> tiled workspace, weights conj(L[c])^T.  The eight
// blocks' values of 32 rows x 16 inputs come in as 64-byte pieces and are laid out in LDS as one plane per block,
// [row][16 + 1]; a wave takes its operands from its own plane.  Four (P = 64) such chunks make a tile; the next
// chunk is fetched into registers while the current one is multiplied.  A wave takes kMTilesPerWaveGather M tiles (see
// cscatter8_kernel).  EMIT: the workgroups of M tile 0 also write
// the chunk to the workspace in the tiled order (dW[row tile][block][l][32 rows]), the operand of the weight-gradient
// kernel, which then does not have to gather dy again.
template <int P>
struct Gather8 {
    static constexpr int kPlane = kRT * 17 + 1;
    static constexpr size_t kLds = 2 * (size_t)8 * kPlane * sizeof(float2);
};

// REAL (see cstage_kernel): the pieces of dy are 32 bytes (eight blocks' values of one (row, input)), a chunk is
// 32 inputs = 16 pairs, and the weights are L[c]^T as stored.
template <int P, int Q, bool EMIT, bool REAL = false>
__global__ void __launch_bounds__(512)
cgather8_kernel(const float2* __restrict__ in, const float2* __restrict__ W, float2* __restrict__ out,
                float2* __restrict__ dwt, int64_t B, int k, int nsplit, int perm_b)
{
    constexpr int MTW = kMTilesPerWaveGather<Q, REAL>;
    constexpr int MTG = Q / 16 / MTW;
    constexpr int NCHUNK = P / 16;
    constexpr int PLANE = Gather8<P>::kPlane;
    extern __shared__ __align__(16) float2 gat8[];

    int bid = (int)blockIdx.x;
    const int split = bid % nsplit;
    bid /= nsplit;
    const int mt0 = (bid % MTG) * MTW, oct = bid / MTG;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g = 8 * oct + w;
    const int col = lane & 31, kh = lane >> 5, e = lane & 1;
    const int64_t ntiles = (B + kRT - 1) / kRT;
    const int64_t ld_in = (int64_t)k * P;
    const bool pb = perm_b != 0;

    float A0[MTW][P / 2], A1[MTW][P / 2];
#pragma unroll
    for (int m = 0; m < MTW; ++m) {
        if constexpr (REAL) {
            const float* Wf = reinterpret_cast<const float*>(W) + (size_t)g * (4 * P * Q) + 32 * (mt0 + m) + col;
#pragma unroll
            for (int u = 0; u < P / 2; ++u) {
                A0[m][u] = Wf[(size_t)(2 * (2 * u + kh)) * (2 * Q)];
                A1[m][u] = Wf[(size_t)(2 * (2 * u + kh) + 1) * (2 * Q)];
            }
        } else {
            const int jw = 16 * (mt0 + m) + (col >> 1);
            const float2* Wg = W + (size_t)g * P * Q;
#pragma unroll
            for (int u = 0; u < P / 2; ++u) {
                const float2 wv = Wg[(2 * u + kh) * Q + jw];
                A0[m][u] = e ? -wv.y : wv.x;
                A1[m][u] = e ? wv.x : wv.y;
            }
        }
    }
    u32x4 pre[4];
    auto fetch = [&](int64_t rt, int ch) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int idx = tid + n * 512;
            const int64_t row = rt * kRT + (idx >> 6);
            if constexpr (REAL) {
                const int part = idx & 1, il = (idx >> 1) & 31;
                const float* srcf = reinterpret_cast<const float*>(in);
                pre[n] = row < B ? ldg128(srcf + row * (2 * ld_in) + (size_t)(32 * ch + il) * k + 8 * oct + 4 * part) : u32x4{0, 0, 0, 0};
            } else {
                const int c2 = idx & 3, ll = (idx >> 2) & 15;
                pre[n] = row < B ? ldg128(in + row * ld_in + (size_t)(16 * ch + ll) * k + 8 * oct + 2 * c2) : u32x4{0, 0, 0, 0};
            }
        }
    };
    auto to_lds = [&](float2* buf) {
#pragma unroll
        for (int n = 0; n < 4; ++n) {
            const int idx = tid + n * 512, r = idx >> 6;
            if constexpr (REAL) {
                const int part = idx & 1, il = (idx >> 1) & 31;
                float* bf = reinterpret_cast<float*>(buf);
#pragma unroll
                for (int t = 0; t < 4; ++t) bf[(4 * part + t) * (2 * PLANE) + r * 34 + il] = __uint_as_float(pre[n][t]);
            } else {
                const int c2 = idx & 3, ll = (idx >> 2) & 15;
                buf[(2 * c2) * PLANE + r * 17 + ll] = make_float2(__uint_as_float(pre[n].x), __uint_as_float(pre[n].y));
                buf[(2 * c2 + 1) * PLANE + r * 17 + ll] = make_float2(__uint_as_float(pre[n].z), __uint_as_float(pre[n].w));
            }
        }
    };

    int64_t rt = split;
    if (rt < ntiles) fetch(rt, 0);
    int cnt = 0;
    for (; rt < ntiles; rt += nsplit) {
        f32x16 acc[MTW];
#pragma unroll
        for (int m = 0; m < MTW; ++m)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[m][r] = 0.f;
#pragma unroll
        for (int ch = 0; ch < NCHUNK; ++ch, ++cnt) {
            float2* buf = gat8 + (cnt & 1) * (8 * PLANE);
            to_lds(buf);
            lds_barrier();
            if (ch + 1 < NCHUNK) fetch(rt, ch + 1);
            else if (rt + nsplit < ntiles) fetch(rt + nsplit, 0);
            const float2* mine = buf + w * PLANE;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float2 xv = mine[col * 17 + 2 * u + kh];
#pragma unroll
                for (int m = 0; m < MTW; ++m) {
                    acc[m] = mfma_f32(A0[m][ch * 8 + u], xv.x, acc[m]);
                    acc[m] = mfma_f32(A1[m][ch * 8 + u], xv.y, acc[m]);
                }
            }
            if constexpr (EMIT) {
                if (mt0 == 0) {
                    float2* dst = dwt + (((size_t)rt * k + g) * P + 16 * ch) * kRT;
#pragma unroll
                    for (int n = 0; n < 8; ++n) dst[(2 * n + kh) * kRT + col] = mine[col * 17 + 2 * n + kh];
                }
            }
        }
#pragma unroll
        for (int m = 0; m < MTW; ++m) {
            if constexpr (REAL) {
                float* outf = reinterpret_cast<float*>(out);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int n = 32 * (mt0 + m) + 8 * (r / 4) + 4 * kh + (r % 4);
                    const int d = mid_src(g * 2 * Q + n, k, 2 * Q, pb);
                    const int blk = d / (2 * Q), idx = d - blk * (2 * Q);
                    outf[((((size_t)rt * k + blk) * Q + (idx >> 1)) * kRT + col) * 2 + (idx & 1)] = acc[m][r];
                }
            } else {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int j = 16 * (mt0 + m) + 4 * q4 + 2 * kh + h;
                        const int d = mid_src(g * Q + j, k, Q, pb);
                        const int blk = d / Q, idx = d - blk * Q;
                        out[(((size_t)rt * k + blk) * Q + idx) * kRT + col] =
                            make_float2(acc[m][4 * q4 + 2 * h], acc[m][4 * q4 + 2 * h + 1]);
                    }
            }
        }
    }
}

// part[z][g][ma][nb] = sum over the rows b of the tiles z, z + Z, ... of  A[b][g][ma] * conj(Bv[b][g][nb])
// A: dW (kInGather from dy) or dY1 (kInT);  Bv: U (kInT) or x (kInNat).  M = 2*MA real rows (re and im of the
// result), N = NB columns, K = (row, component): with B'[(b,t)][nb] = component t of Bv[b][nb],
//   A'[2ma][(b,0)] = ar,  A'[2ma][(b,1)] = ai,  A'[2ma+1][(b,0)] = ai,  A'[2ma+1][(b,1)] = -ar.
// Wave w owns the 16 values ma = 16w .. 16w+15 and every column.  LDS holds each operand so that the lanes of a
// wave read consecutive addresses for one row: [row][len] for row-major sources, [idx][32 + 1] for the tiled ones.
template <int LEN, int NTHR, int MODE, bool REAL = false>
struct WgTile {
    static constexpr int kPieces = (MODE == kInGather) ? kRT * LEN / NTHR : kRT * LEN / 2 / NTHR;
    static constexpr int kLen = (MODE == kInT) ? LEN * (kRT + 1) : kRT * LEN;
    u32x4 v[MODE == kInGather ? (kPieces + 1) / 2 : kPieces];

    __device__ __forceinline__ void fetch(const float2* __restrict__ src, int64_t rt, int g, int k, int64_t ld, int64_t B, int tid)
    {
        const int64_t row0 = rt * kRT;
        if constexpr (MODE == kInNat) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / (LEN / 2), c2 = idx - row * (LEN / 2);
                v[n] = (row0 + row < B) ? ldg128(src + (row0 + row) * ld + (size_t)g * LEN + 2 * c2) : u32x4{0, 0, 0, 0};
            }
        } else if constexpr (MODE == kInGather && REAL) {
            const float* srcf = reinterpret_cast<const float*>(src);
#pragma unroll
            for (int n = 0; n < 2 * kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / (2 * LEN), i = idx - row * (2 * LEN);
                float t = 0.f;
                if (row0 + row < B) t = srcf[(row0 + row) * (2 * ld) + (size_t)i * k + g];
                v[n / 4][n % 4] = __float_as_uint(t);
            }
        } else if constexpr (MODE == kInGather) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, row = idx / LEN, i = idx - row * LEN;
                float2 t = make_float2(0.f, 0.f);
                if (row0 + row < B) t = src[(row0 + row) * ld + (size_t)i * k + g];
                if (n & 1) { v[n / 2].z = __float_as_uint(t.x); v[n / 2].w = __float_as_uint(t.y); }
                else { v[n / 2].x = __float_as_uint(t.x); v[n / 2].y = __float_as_uint(t.y); }
            }
        } else {
            const float2* tile = src + ((size_t)rt * k + g) * (LEN * kRT);
#pragma unroll
            for (int n = 0; n < kPieces; ++n) v[n] = ldg128(tile + 2 * (tid + n * NTHR));
        }
    }

    __device__ __forceinline__ void to_lds(float2* t, int tid) const
    {
        if constexpr (MODE == kInNat) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) *reinterpret_cast<u32x4*>(t + 2 * (tid + n * NTHR)) = v[n];
        } else if constexpr (MODE == kInGather && REAL) {
            float* tf = reinterpret_cast<float*>(t);
#pragma unroll
            for (int n = 0; n < 2 * kPieces; ++n) tf[tid + n * NTHR] = __uint_as_float(v[n / 4][n % 4]);
        } else if constexpr (MODE == kInGather) {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const u32x4 w = v[n / 2];
                t[tid + n * NTHR] = (n & 1) ? make_float2(__uint_as_float(w.z), __uint_as_float(w.w))
                                            : make_float2(__uint_as_float(w.x), __uint_as_float(w.y));
            }
        } else {
#pragma unroll
            for (int n = 0; n < kPieces; ++n) {
                const int idx = tid + n * NTHR, i = idx / (kRT / 2), rp = idx - i * (kRT / 2);
                lds_store_c2(t + i * (kRT + 1) + 2 * rp, v[n]);
            }
        }
    }

    static __device__ __forceinline__ float2 at(const float2* t, int idx, int row)
    {
        return (MODE == kInT) ? t[idx * (kRT + 1) + row] : t[row * LEN + idx];
    }
};

// REAL: real fp32 operands, two consecutive values per float2: out[g][ma'][nb'] = sum_b A[b][g][ma'] * Bv[b][g][nb'] for
// the 2*MA x 2*NB real indices; a K = 2 step contracts two batch rows, each lane picking its component of the pair.
template <int MA, int NB, int AMODE, int BMODE, bool REAL = false>
__global__ void __launch_bounds__(4 * MA)
cwgrad_kernel(const float2* __restrict__ A, const float2* __restrict__ Bv, float2* __restrict__ part, int64_t B, int k,
              int Z, int64_t lda, int64_t ldb)
{
    constexpr int NTHR = 4 * MA;
    constexpr int NTN = REAL ? (2 * NB + 31) / 32 : (NB + 31) / 32;
    using TA = WgTile<MA, NTHR, AMODE, REAL>;
    using TB = WgTile<NB, NTHR, BMODE, REAL>;
    extern __shared__ __align__(16) float2 wg_lds[];  // two buffers of each operand: 2 * (TA::kLen + TB::kLen) values

    const int g = (int)blockIdx.x / Z, z = (int)blockIdx.x - g * Z;
    const int tid = threadIdx.x, lane = tid & 63, mt = tid >> 6;
    const int col = lane & 31, kh = lane >> 5, e = lane & 1;
    const int ma = 16 * mt + (col >> 1);
    const int64_t ntiles = (B + kRT - 1) / kRT;

    f32x16 acc[NTN];
#pragma unroll
    for (int nt = 0; nt < NTN; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;

    TA pa;
    TB pbv;
    int64_t rt = z;
    if (rt < ntiles) {
        pa.fetch(A, rt, g, k, lda, B, tid);
        pbv.fetch(Bv, rt, g, k, ldb, B, tid);
    }
    for (int it = 0; rt < ntiles; rt += Z, ++it) {
        float2* ta = wg_lds + (it & 1) * TA::kLen;
        float2* tb = wg_lds + 2 * TA::kLen + (it & 1) * TB::kLen;
        pa.to_lds(ta, tid);
        pbv.to_lds(tb, tid);
        lds_barrier();
        if (rt + Z < ntiles) {
            pa.fetch(A, rt + Z, g, k, lda, B, tid);
            pbv.fetch(Bv, rt + Z, g, k, ldb, B, tid);
        }
#pragma unroll
        for (int u = 0; u < kRT / 2; ++u) {
            const int b = 2 * u + kh;
            const float2 av = TA::at(ta, ma, b);
            if constexpr (REAL) {
                const float as = e ? av.y : av.x;
#pragma unroll
                for (int nt = 0; nt < NTN; ++nt) {
                    const int nbp = 16 * nt + (col >> 1);  // the pair holding real column 32*nt + col
                    const float2 bv = (NB % 16 == 0 || nbp < NB) ? TB::at(tb, nbp, b) : make_float2(0.f, 0.f);
                    acc[nt] = mfma_f32(as, e ? bv.y : bv.x, acc[nt]);
                }
            } else {
                const float a0 = e ? av.y : av.x;
                const float a1 = e ? -av.x : av.y;
#pragma unroll
                for (int nt = 0; nt < NTN; ++nt) {
                    const int nb = 32 * nt + col;
                    const float2 bv = (NB % 32 == 0 || nb < NB) ? TB::at(tb, nb, b) : make_float2(0.f, 0.f);
                    acc[nt] = mfma_f32(a0, bv.x, acc[nt]);
                    acc[nt] = mfma_f32(a1, bv.y, acc[nt]);
                }
            }
        }
    }
    if constexpr (REAL) {
        // acc[nt][r]: row 32*mt + 8*(r/4) + 4*kh + r%4, column 32*nt + col of the (2*MA) x (2*NB) block
        float* o = reinterpret_cast<float*>(part) + ((size_t)z * k + g) * (4 * MA * NB);
#pragma unroll
        for (int nt = 0; nt < NTN; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                o[(size_t)(32 * mt + 8 * (r / 4) + 4 * kh + (r % 4)) * (2 * NB) + 32 * nt + col] = acc[nt][r];
    } else {
        float2* o = part + ((size_t)z * k + g) * (MA * NB);
#pragma unroll
        for (int nt = 0; nt < NTN; ++nt) {
            const int nb = 32 * nt + col;
            if (NB % 32 != 0 && nb >= NB) continue;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    o[(16 * mt + 4 * q4 + 2 * kh + h) * NB + nb] = make_float2(acc[nt][4 * q4 + 2 * h], acc[nt][4 * q4 + 2 * h + 1]);
        }
    }
}

// out[e] = part[0][e] + part[1][e] + ... + part[Z-1][e], in that order; e counts float4s
__global__ void __launch_bounds__(256) csum_kernel(const f32x4* __restrict__ part, f32x4* __restrict__ out, size_t n4, int Z)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n4) return;
    f32x4 s = part[e];
    int z = 1;
    for (; z + 8 <= Z; z += 8) {  // eight loads in flight, added in order
        f32x4 t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = part[(size_t)(z + u) * n4 + e];
#pragma unroll
        for (int u = 0; u < 8; ++u) { s.x += t[u].x; s.y += t[u].y; s.z += t[u].z; s.w += t[u].w; }
    }
    for (; z < Z; ++z) {
        const f32x4 t = part[(size_t)z * n4 + e];
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    out[e] = s;
}

int64_t tiles_of(const Problem& pb) { return (pb.B + kRT - 1) / kRT; }
size_t t_bytes(const Problem& pb) { return align_up((size_t)tiles_of(pb) * kRT * pb.kq() * sizeof(float2), 256); }

// workgroups of one block: enough for about sixteen waves per CU in all, a multiple of 8, at most one per tile
int splits_for(const Problem& pb, int waves_per_wg, int target_waves)
{
    int64_t n = (target_waves / waves_per_wg + pb.k - 1) / pb.k;
    n = (n + 7) / 8 * 8;
    const int64_t t = tiles_of(pb);
    if (n > t) n = t;
    return (int)(n < 1 ? 1 : n);
}

int wgrad_chunks(const Problem& pb)
{
    int64_t z = (512 + pb.k - 1) / pb.k;
    z = (z + 7) / 8 * 8;
    const int64_t t = tiles_of(pb);
    if (z > t) z = t;
    return (int)(z < 1 ? 1 : z);
}

template <int M, int IN, int OUT, bool CONJT, bool REAL = false>
int launch_stage(const Problem& pb, const void* in, const void* W, void* out, hipStream_t st)
{
    const int nsplit = splits_for(pb, M / 16, 4096);
    const int64_t grid = (int64_t)pb.k * nsplit;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL((cstage_kernel<M, M, IN, OUT, CONJT, REAL>), dim3((unsigned)grid), dim3(4 * M), 0, st, (const float2*)in,
                       (const float2*)W, (float2*)out, pb.B, pb.k, nsplit, pb.perm_b() ? 1 : 0);
    return hip_status(hipGetLastError());
}

// the eight-blocks-per-workgroup stages: about two workgroups per CU, a multiple of 8 per (block octet, M tile)
int splits8_for(const Problem& pb, int mtiles)
{
    int64_t n = (512 + (pb.k / 8) * mtiles - 1) / ((pb.k / 8) * mtiles);
    n = (n + 7) / 8 * 8;
    const int64_t t = tiles_of(pb);
    if (n > t) n = t;
    return (int)(n < 1 ? 1 : n);
}

template <int M, bool REAL = false>
int launch_scatter8(const Problem& pb, const void* T, const void* W, void* out, hipStream_t st)
{
    constexpr int MTG = M / 16 / Scatter8<M, M>::MTW;
    const int nsplit = splits8_for(pb, MTG);
    const int64_t grid = (int64_t)(pb.k / 8) * MTG * nsplit;
    if (grid > 0x7fffffffLL) return -2;
    auto kern = cscatter8_kernel<M, M, REAL>;
    constexpr size_t lds = Scatter8<M, M>::kLds;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), lds, st, (const float2*)T, (const float2*)W,
                       (float2*)out, pb.B, pb.k, nsplit);
    return hip_status(hipGetLastError());
}

template <int M, bool EMIT, bool REAL = false>
int launch_gather8(const Problem& pb, const void* in, const void* W, void* out, void* dwt, hipStream_t st)
{
    constexpr int MTG = M / 16 / kMTilesPerWaveGather<M, REAL>;
    const int nsplit = splits8_for(pb, MTG);
    const int64_t grid = (int64_t)(pb.k / 8) * MTG * nsplit;
    if (grid > 0x7fffffffLL) return -2;
    auto kern = cgather8_kernel<M, M, EMIT, REAL>;
    constexpr size_t lds = Gather8<M>::kLds;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), lds, st, (const float2*)in, (const float2*)W,
                       (float2*)out, (float2*)dwt, pb.B, pb.k, nsplit, pb.perm_b() ? 1 : 0);
    return hip_status(hipGetLastError());
}

// lda, ldb: row lengths of row-major operands in float2 units
template <int M, int AMODE, int BMODE, bool REAL = false>
int launch_wgrad(const Problem& pb, const void* A, const void* Bv, void* out, void* part, int64_t lda, int64_t ldb,
                 hipStream_t st)
{
    const int Z = wgrad_chunks(pb);
    const int64_t grid = (int64_t)pb.k * Z;
    if (grid > 0x7fffffffLL) return -2;
    float2* dst = Z == 1 ? (float2*)out : (float2*)part;
    auto kern = cwgrad_kernel<M, M, AMODE, BMODE, REAL>;
    const size_t lds = 2 * (size_t)(WgTile<M, 4 * M, AMODE, REAL>::kLen + WgTile<M, 4 * M, BMODE, REAL>::kLen) * sizeof(float2);
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(4 * M), lds, st, (const float2*)A, (const float2*)Bv, dst, pb.B,
                       pb.k, Z, lda, ldb);
    int rc = hip_status(hipGetLastError());
    if (rc || Z == 1) return rc;
    const size_t n4 = (size_t)pb.k * M * M / (REAL ? 1 : 2);  // float4s of one gradient: (2M)^2 floats, or M^2 complex values, per block
    hipLaunchKernelGGL(csum_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, (const f32x4*)part, (f32x4*)out, n4, Z);
    return hip_status(hipGetLastError());
}

template <int M>
int run_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    int rc = launch_stage<M, kInNat, kOutTFwd, false>(pb, x, R, ws, st);
    if (rc) return rc;
    if (pb.k % 8 == 0) return launch_scatter8<M>(pb, ws, L, y, st);
    return launch_stage<M, kInT, kOutScatter, false>(pb, ws, L, y, st);
}

template <int M>
int run_fwd_h(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    int rc = pb.k % 8 == 0 ? launch_gather8<M, false>(pb, x, L, ws, nullptr, st)
                           : launch_stage<M, kInGather, kOutTBwd, true>(pb, x, L, ws, st);
    if (rc) return rc;
    return launch_stage<M, kInT, kOutNat, true>(pb, ws, R, y, st);
}

template <int M>
int run_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR, void* dL,
            void* ws, hipStream_t st)
{
    char* w = (char*)ws;
    void* Ut = w;
    void* dY1t = w + t_bytes(pb);
    void* dWt = w + 2 * t_bytes(pb);
    void* part = w + 3 * t_bytes(pb);
    const bool eight = pb.k % 8 == 0;
    int rc = launch_stage<M, kInNat, kOutTFwd, false>(pb, x, R, Ut, st);
    if (rc) return rc;
    rc = eight ? launch_gather8<M, true>(pb, dy, L, dY1t, dWt, st) : launch_stage<M, kInGather, kOutTBwd, true>(pb, dy, L, dY1t, st);
    if (rc) return rc;
    rc = launch_stage<M, kInT, kOutNat, true>(pb, dY1t, R, dx, st);
    if (rc) return rc;
    rc = eight ? launch_wgrad<M, kInT, kInT>(pb, dWt, Ut, dL, part, 0, 0, st)
               : launch_wgrad<M, kInGather, kInT>(pb, dy, Ut, dL, part, pb.n_out(), 0, st);
    if (rc) return rc;
    return launch_wgrad<M, kInT, kInNat>(pb, dY1t, x, dR, part, 0, pb.n_in, st);
}

// ---- real fp32 layers with square blocks of 32 or 64 on the same kernels (REAL): M = block size / 2 ----
size_t rt_bytes(const Problem& pb) { return align_up((size_t)tiles_of(pb) * kRT * pb.kq() * sizeof(float), 256); }

template <int M>
int run_real_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    int rc = launch_stage<M, kInNat, kOutTFwd, false, true>(pb, x, R, ws, st);
    if (rc) return rc;
    if (pb.k % 8 == 0) return launch_scatter8<M, true>(pb, ws, L, y, st);
    return launch_stage<M, kInT, kOutScatter, false, true>(pb, ws, L, y, st);
}

template <int M>
int run_real_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    int rc = pb.k % 8 == 0 ? launch_gather8<M, false, true>(pb, x, L, ws, nullptr, st)
                           : launch_stage<M, kInGather, kOutTBwd, true, true>(pb, x, L, ws, st);
    if (rc) return rc;
    return launch_stage<M, kInT, kOutNat, true, true>(pb, ws, R, y, st);
}

template <int M>
int run_real_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                 void* dL, void* ws, hipStream_t st)
{
    char* w = (char*)ws;
    void* Ut = w;
    void* dY1t = w + rt_bytes(pb);
    void* dWt = w + 2 * rt_bytes(pb);
    void* part = w + 3 * rt_bytes(pb);
    const bool eight = pb.k % 8 == 0;
    int rc = launch_stage<M, kInNat, kOutTFwd, false, true>(pb, x, R, Ut, st);
    if (rc) return rc;
    rc = eight ? launch_gather8<M, true, true>(pb, dy, L, dY1t, dWt, st)
               : launch_stage<M, kInGather, kOutTBwd, true, true>(pb, dy, L, dY1t, st);
    if (rc) return rc;
    rc = launch_stage<M, kInT, kOutNat, true, true>(pb, dY1t, R, dx, st);
    if (rc) return rc;
    rc = eight ? launch_wgrad<M, kInT, kInT, true>(pb, dWt, Ut, dL, part, 0, 0, st)
               : launch_wgrad<M, kInGather, kInT, true>(pb, dy, Ut, dL, part, pb.n_out() / 2, 0, st);
    if (rc) return rc;
    return launch_wgrad<M, kInT, kInNat, true>(pb, dY1t, x, dR, part, 0, pb.n_in / 2, st);
}

}  // namespace

bool real32_mfma_supported(const Problem& pb)
{
    return pb.dtype == 0 && pb.p == pb.q && pb.q == pb.s && (pb.p == 32 || pb.p == 64);
}

// pass: 0 forward, 1 backward, 2 transposed multiply
size_t real32_mfma_workspace(const Problem& pb, int pass)
{
    if (pass != 1) return rt_bytes(pb);
    const int Z = wgrad_chunks(pb);
    return 3 * rt_bytes(pb) + (Z > 1 ? align_up((size_t)Z * pb.n_L() * sizeof(float), 256) : 0);
}

int real32_mfma_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    return pb.p == 32 ? run_real_fwd<16>(pb, x, R, L, y, ws, st) : run_real_fwd<32>(pb, x, R, L, y, ws, st);
}

int real32_mfma_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    return pb.p == 32 ? run_real_fwd_t<16>(pb, x, R, L, y, ws, st) : run_real_fwd_t<32>(pb, x, R, L, y, ws, st);
}

int real32_mfma_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                    void* dL, void* ws, hipStream_t st)
{
    if (pb.B == 0) {
        const int rc = launch_fill_zero_f32((float*)dR, pb.n_R(), st);
        return rc ? rc : launch_fill_zero_f32((float*)dL, pb.n_L(), st);
    }
    return pb.p == 32 ? run_real_bwd<16>(pb, dy, x, R, L, dx, dR, dL, ws, st) : run_real_bwd<32>(pb, dy, x, R, L, dx, dR, dL, ws, st);
}

bool complex_mfma_supported(const Problem& pb)
{
    return pb.p == pb.q && pb.q == pb.s && (pb.p == 16 || pb.p == 32 || pb.p == 64);
}

// pass: 0 forward, 1 backward, 2 conjugate-transpose forward
size_t complex_mfma_workspace(const Problem& pb, int pass)
{
    if (pass != 1) return t_bytes(pb);
    const int Z = wgrad_chunks(pb);
    return 3 * t_bytes(pb) + (Z > 1 ? align_up((size_t)Z * pb.n_L() * sizeof(float2), 256) : 0);
}

int complex_mfma_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    switch (pb.p) {
        case 16: return run_fwd<16>(pb, x, R, L, y, ws, st);
        case 32: return run_fwd<32>(pb, x, R, L, y, ws, st);
        case 64: return run_fwd<64>(pb, x, R, L, y, ws, st);
        default: return -2;
    }
}

int complex_mfma_fwd_h(const Problem& pb, const void* x, const void* R, const void* L, void* y, void* ws, hipStream_t st)
{
    switch (pb.p) {
        case 16: return run_fwd_h<16>(pb, x, R, L, y, ws, st);
        case 32: return run_fwd_h<32>(pb, x, R, L, y, ws, st);
        case 64: return run_fwd_h<64>(pb, x, R, L, y, ws, st);
        default: return -2;
    }
}

int complex_mfma_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                     void* dL, void* ws, hipStream_t st)
{
    switch (pb.p) {
        case 16: return run_bwd<16>(pb, dy, x, R, L, dx, dR, dL, ws, st);
        case 32: return run_bwd<32>(pb, dy, x, R, L, dx, dR, dL, ws, st);
        case 64: return run_bwd<64>(pb, dy, x, R, L, dx, dR, dL, ws, st);
        default: return -2;
    }
}

}  // namespace monarch
