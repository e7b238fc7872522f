// Column sums of the upstream gradient (the bias gradient dbias[o] = sum_b dy[b][o]) as device
// bodies, so that the two passes can run either as kernels of their own or as extra workgroups at the
// tail of launches the backward makes anyway (the weight re-layout and the weight-gradient reduction).
#pragma once
#include "monarch_device.h"

namespace monarch {

// CW consecutive elements of one row as fp32: one 8/16-byte access for CW = 4.
template <typename T, int CW> struct ColVec;
template <> struct ColVec<float, 1> {
    static __device__ __forceinline__ void load(const float* p, float* v) { v[0] = *p; }
    static __device__ __forceinline__ void store(float* p, const float* v) { *p = v[0]; }
};
template <> struct ColVec<bf16_t, 1> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* v) { v[0] = bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, const float* v) { *p = f32_to_bf16(v[0]); }
};
template <> struct ColVec<float, 4> {
    static __device__ __forceinline__ void load(const float* p, float* v)
    {
        const float4 t = *(const float4*)p;
        v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
    }
    static __device__ __forceinline__ void store(float* p, const float* v) { *(float4*)p = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct ColVec<bf16_t, 4> {
    static __device__ __forceinline__ void load(const bf16_t* p, float* v)
    {
        const uint2 t = *(const uint2*)p;
        v[0] = __uint_as_float(t.x << 16), v[1] = __uint_as_float(t.x & 0xffff0000u);
        v[2] = __uint_as_float(t.y << 16), v[3] = __uint_as_float(t.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float* v)
    {
        uint2 t;
        t.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
        t.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
        *(uint2*)p = t;
    }
};


// dy is walked as (row chunk) x (tile of 64 * CW columns): a workgroup is four waves, wave w takes rows
// w, w + 4, ... of the chunk, four rows at a time so that four independent 8/16-byte loads are in
// flight per lane, and a lane owns CW consecutive columns (CW = 4 when 4 divides n_out, else 1).  The
// chunk count is chosen for about a thousand workgroups with at least 16 rows each.
constexpr int ROWCOL_WAVES = 4;
constexpr int ROWCOL_MAX_CHUNKS = 1024;

static inline int rowcol_cw(int n_out) { return n_out % 4 == 0 ? 4 : 1; }
static inline int rowcol_col_tiles(int n_out) { return (n_out / rowcol_cw(n_out) + 63) / 64; }
static inline int rowcol_chunks(int64_t B, int n_out)
{
    int64_t c = (B + 15) / 16;
    const int64_t cap = ROWCOL_MAX_CHUNKS / rowcol_col_tiles(n_out) > 0 ? ROWCOL_MAX_CHUNKS / rowcol_col_tiles(n_out) : 1;
    if (c > cap) c = cap;
    return c < 1 ? 1 : (int)c;
}


struct ColsumJob {
    const void* dy;  // (B, n_out)
    float* part;     // chunks x n_out fp32 partial rows
    void* dbias;     // n_out, fp32 or bf16
    int64_t B;
    int n_out, col_tiles, chunks, out_f32;
};

static inline int colsum_partial_blocks(const ColsumJob& cj) { return cj.col_tiles * cj.chunks; }
static inline int colsum_final_blocks(const ColsumJob& cj) { return (cj.n_out + 63) / 64; }

// Pass 1, workgroup `block` of colsum_partial_blocks (256 threads): each wave adds its rows of the
// chunk in fp32, the four waves meet in LDS, wave 0 adds them in wave order and writes one fp32 partial
// row per chunk.  Every thread of the workgroup must call it (it contains a barrier).
template <typename T, int CW>
__device__ __forceinline__ void colsum_partial_body(const ColsumJob& cj, int block)
{
    __shared__ float red[ROWCOL_WAVES - 1][CW][64];
    const T* __restrict__ dy = (const T*)cj.dy;
    const int n_out = cj.n_out;
    const int ct = block % cj.col_tiles, ch = block / cj.col_tiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = (ct * 64 + lane) * CW;
    const bool live = col < n_out;
    const int64_t rows_per = (cj.B + cj.chunks - 1) / cj.chunks;
    const int64_t r0 = ch * rows_per;
    int64_t r1 = r0 + rows_per;
    if (r1 > cj.B) r1 = cj.B;
    if (!live) r1 = r0;
    float acc[4][CW];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < CW; ++e) acc[u][e] = 0.f;
    int64_t r = r0 + wave;
    for (; r + 3 * ROWCOL_WAVES < r1; r += 4 * ROWCOL_WAVES) {
        float v[4][CW];
#pragma unroll
        for (int u = 0; u < 4; ++u) ColVec<T, CW>::load(dy + (size_t)(r + u * ROWCOL_WAVES) * n_out + col, v[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int e = 0; e < CW; ++e) acc[u][e] += v[u][e];
    }
    for (; r < r1; r += ROWCOL_WAVES) {
        float v[CW];
        ColVec<T, CW>::load(dy + (size_t)r * n_out + col, v);
#pragma unroll
        for (int e = 0; e < CW; ++e) acc[0][e] += v[e];
    }
    float sum[CW];
#pragma unroll
    for (int e = 0; e < CW; ++e) sum[e] = (acc[0][e] + acc[1][e]) + (acc[2][e] + acc[3][e]);
    if (wave > 0) {
#pragma unroll
        for (int e = 0; e < CW; ++e) red[wave - 1][e][lane] = sum[e];
    }
    __syncthreads();
    if (wave > 0 || !live) return;
#pragma unroll
    for (int w = 0; w < ROWCOL_WAVES - 1; ++w)
#pragma unroll
        for (int e = 0; e < CW; ++e) sum[e] += red[w][e][lane];
#pragma unroll
    for (int e = 0; e < CW; ++e) cj.part[(size_t)ch * n_out + col + e] = sum[e];
}

// Pass 2, workgroup `block` of colsum_final_blocks (64 * NL threads): the workgroup owns 64 columns;
// NL groups of lanes each add every NL-th chunk partial, the NL sums meet in LDS and are added in
// order; one rounding to the output type.  Every thread of the workgroup must call it.
template <typename TO, int NL>
__device__ __forceinline__ void colsum_final_body(const ColsumJob& cj, int block)
{
    __shared__ float red[NL][64];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int o = block * 64 + tx;
    float acc = 0.f;
    if (o < cj.n_out) {
#pragma unroll 4
        for (int ch = ty; ch < cj.chunks; ch += NL) acc += cj.part[(size_t)ch * cj.n_out + o];
    }
    red[ty][tx] = acc;
    __syncthreads();
    if (ty > 0 || o >= cj.n_out) return;
    acc = 0.f;
#pragma unroll
    for (int w = 0; w < NL; ++w) acc += red[w][tx];
    Elem<TO>::store((TO*)cj.dbias + o, acc);
}

}  // namespace monarch
