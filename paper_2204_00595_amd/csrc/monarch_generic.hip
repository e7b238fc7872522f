// Shape-generic fused kernels for the Monarch multiply: any k, p, q, s, fp32 or bf16
// storage, both readings of the mid permutation.  They are the fallback for shapes the
// MFMA kernels do not cover; plain fp32 FMA, one workgroup per tile of BM batch rows,
// the intermediate (Y1 / U of Section 3.3) lives in LDS only.
#include "monarch_internal.h"
#include "monarch_device.h"
#include "monarch_colsum.h"

namespace monarch {

static constexpr int kThreads = 256;

// ------------------------------------------------------------------ utilities ----

__global__ void fill_zero_f32_kernel(float* p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0.f;
}

__global__ void fill_zero_u16_kernel(uint16_t* p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0;
}

__global__ void f32_to_bf16_kernel(const float* src, uint16_t* dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = f32_to_bf16(src[i]);
}

static int grid_for(size_t n)
{
    size_t g = (n + kThreads - 1) / kThreads;
    if (g > 2048) g = 2048;
    if (g < 1) g = 1;
    return (int)g;
}

// Streaming copy: one workgroup per 16 KiB segment, four independent 16-byte non-temporal loads in
// flight per lane, non-temporal stores (measured: 6.0 TB/s for 1 GiB on MI355X, against 4.5 TB/s with
// ordinary loads and stores in a grid-stride loop).
typedef __attribute__((ext_vector_type(4))) unsigned int copy_v4;

__global__ void __launch_bounds__(256) stream_copy_kernel(copy_v4* __restrict__ dst, const copy_v4* __restrict__ src, size_t n16)
{
    const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
    if (i + 768 < n16) {
        const copy_v4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + 256),
                      c = __builtin_nontemporal_load(src + i + 512), d = __builtin_nontemporal_load(src + i + 768);
        __builtin_nontemporal_store(a, dst + i);
        __builtin_nontemporal_store(b, dst + i + 256);
        __builtin_nontemporal_store(c, dst + i + 512);
        __builtin_nontemporal_store(d, dst + i + 768);
    } else {
        for (size_t j = i; j < n16 && j < i + 1024; j += 256) __builtin_nontemporal_store(__builtin_nontemporal_load(src + j), dst + j);
    }
}

int launch_stream_copy(void* dst, const void* src, size_t nbytes, hipStream_t st)
{
    const size_t n16 = nbytes / 16;
    if (n16 == 0) return 0;
    const size_t grid = (n16 + 1023) / 1024;
    if (grid > 0x7fffffffULL) return -2;
    hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)grid), dim3(256), 0, st, (copy_v4*)dst, (const copy_v4*)src, n16);
    return hip_status(hipGetLastError());
}

int launch_fill_zero_f32(float* p, size_t n, hipStream_t st)
{
    if (n == 0) return 0;
    hipLaunchKernelGGL(fill_zero_f32_kernel, dim3(grid_for(n)), dim3(kThreads), 0, st, p, n);
    return hip_status(hipGetLastError());
}

int launch_fill_zero_u16(uint16_t* p, size_t n, hipStream_t st)
{
    if (n == 0) return 0;
    hipLaunchKernelGGL(fill_zero_u16_kernel, dim3(grid_for(n)), dim3(kThreads), 0, st, p, n);
    return hip_status(hipGetLastError());
}

int launch_f32_to_bf16(const float* src, uint16_t* dst, size_t n, hipStream_t st)
{
    if (n == 0) return 0;
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(grid_for(n)), dim3(kThreads), 0, st, src, dst, n);
    return hip_status(hipGetLastError());
}

// ------------------------------------------------------------- dense form of M ----
//
// Entry (o, col) of M = P L P^T R with o = l*k + c and col = kk*p + i is the sum, over the stage-1
// outputs j of block kk that the mid permutation sends into block c of stage 2 (position r there),
// of L[c][l][r] * R[kk][j][i]: one term in the square case (Equation (1)), about q/k terms otherwise.
// In the default reading those j are a contiguous range (g = j*k + kk must fall in [c*q, (c+1)*q)),
// in the inverse reading every k-th j (f = kk*q + j must be congruent to c mod k).
// One thread owns CW consecutive columns (CW = 4 when 4 divides p, one 8- or 16-byte load per R row,
// else 1) and DENSE_LT consecutive l of one c, so an R element is loaded once for DENSE_LT outputs;
// lanes of a wave read consecutive i (coalesced) and share the L values.

static constexpr int DENSE_LT = 8;
static constexpr int DENSE_THREADS = 64;

// The DENSE_JS waves of a workgroup share the same outputs and split the terms of the sum between
// them (wave w takes terms w, w + DENSE_JS, ...): a wave's chain of dependent-latency loads is
// DENSE_JS times shorter and a small matrix with long sums still fills the chip (measured, 768 x 768
// with 48 terms per entry: 8.5 us against 15.5 us with one wave; large matrices and single-term sums
// are faster with one wave).  The partial sums meet in LDS and wave 0 adds them in wave order (a
// fixed order: the result is reproducible).
template <typename T, int CW, int DENSE_JS>
__global__ void __launch_bounds__(DENSE_THREADS * DENSE_JS)
to_dense_kernel(const T* __restrict__ R, const T* __restrict__ L, T* __restrict__ M, int k, int p, int q, int s,
                int perm_b, int col_tiles, int l_tiles)
{
    __shared__ float part[DENSE_JS > 1 ? DENSE_JS - 1 : 1][DENSE_LT * CW][DENSE_THREADS];
    const int n_in = k * p;
    const int ct = blockIdx.x % col_tiles;
    const int rest = blockIdx.x / col_tiles;
    const int lt = rest % l_tiles;
    const int c = rest / l_tiles;
    const int lane = threadIdx.x % DENSE_THREADS, wave = threadIdx.x / DENSE_THREADS;
    const int col = (ct * DENSE_THREADS + lane) * CW;  // CW | p, so the CW columns share kk
    const bool live = col < n_in;
    const int kk = live ? col / p : 0, i = live ? col - kk * p : 0;
    const int l0 = lt * DENSE_LT;

    int j0, j1, jstep;
    if (!perm_b) {
        // j*k + kk >= c*q  and  j*k + kk < (c+1)*q
        const int lo = c * q - kk, hi = (c + 1) * q - kk;
        j0 = lo <= 0 ? 0 : (lo + k - 1) / k;
        j1 = hi <= 0 ? 0 : (hi + k - 1) / k;
        if (j1 > q) j1 = q;
        jstep = 1;
    } else {
        // (kk*q + j) mod k == c
        const int base = (int)(((int64_t)kk * q) % k);
        j0 = c - base;
        if (j0 < 0) j0 += k;
        j1 = q;
        jstep = k;
    }
    if (!live) j1 = j0;

    float acc[DENSE_LT][CW];
#pragma unroll
    for (int u = 0; u < DENSE_LT; ++u)
#pragma unroll
        for (int e = 0; e < CW; ++e) acc[u][e] = 0.f;
    const T* Rk = R + (size_t)kk * q * p + i;
    const T* Lc = L + (size_t)c * s * q;
    for (int j = j0 + wave * jstep; j < j1; j += jstep * DENSE_JS) {
        const int r = mid_dest(kk * q + j, k, q, perm_b != 0) - c * q;
        float w[CW];
        ColVec<T, CW>::load(Rk + (size_t)j * p, w);
#pragma unroll
        for (int u = 0; u < DENSE_LT; ++u) {
            const int l = l0 + u < s ? l0 + u : s - 1;
            const float a = Elem<T>::load(Lc + (size_t)l * q + r);
#pragma unroll
            for (int e = 0; e < CW; ++e) acc[u][e] = fmaf(a, w[e], acc[u][e]);
        }
    }
    if (DENSE_JS > 1) {
        if (wave > 0) {
#pragma unroll
            for (int u = 0; u < DENSE_LT; ++u)
#pragma unroll
                for (int e = 0; e < CW; ++e) part[wave - 1][u * CW + e][lane] = acc[u][e];
        }
        __syncthreads();
        if (wave > 0) return;
#pragma unroll
        for (int w2 = 0; w2 < DENSE_JS - 1; ++w2)
#pragma unroll
            for (int u = 0; u < DENSE_LT; ++u)
#pragma unroll
                for (int e = 0; e < CW; ++e) acc[u][e] += part[w2][u * CW + e][lane];
    }
    if (!live) return;
#pragma unroll
    for (int u = 0; u < DENSE_LT; ++u)
        if (l0 + u < s) ColVec<T, CW>::store(M + ((size_t)(l0 + u) * k + c) * n_in + col, acc[u]);
}

template <typename T, int CW, int JS>
static void launch_to_dense_v(const Problem& pb, const void* R, const void* L, void* M, hipStream_t st, unsigned grid,
                              int col_tiles, int l_tiles)
{
    hipLaunchKernelGGL((to_dense_kernel<T, CW, JS>), dim3(grid), dim3(DENSE_THREADS * JS), 0, st, (const T*)R,
                       (const T*)L, (T*)M, pb.k, pb.p, pb.q, pb.s, pb.perm_b() ? 1 : 0, col_tiles, l_tiles);
}

template <typename T>
static int launch_to_dense_t(const Problem& pb, const void* R, const void* L, void* M, hipStream_t st)
{
    const int cw = pb.p % 4 == 0 ? 4 : 1;
    const int col_tiles = (pb.n_in / cw + DENSE_THREADS - 1) / DENSE_THREADS;
    const int l_tiles = (pb.s + DENSE_LT - 1) / DENSE_LT;
    const int64_t grid = (int64_t)col_tiles * l_tiles * pb.k;
    if (grid > 0x7fffffffLL) return -2;
    const bool split = grid < 2048 && pb.q / pb.k >= 16;  // few workgroups, long sums
    const unsigned g = (unsigned)grid;
    if (cw == 4) {
        if (split) launch_to_dense_v<T, 4, 4>(pb, R, L, M, st, g, col_tiles, l_tiles);
        else launch_to_dense_v<T, 4, 1>(pb, R, L, M, st, g, col_tiles, l_tiles);
    } else {
        if (split) launch_to_dense_v<T, 1, 4>(pb, R, L, M, st, g, col_tiles, l_tiles);
        else launch_to_dense_v<T, 1, 1>(pb, R, L, M, st, g, col_tiles, l_tiles);
    }
    return hip_status(hipGetLastError());
}

int launch_to_dense(const Problem& pb, const void* R, const void* L, void* M, hipStream_t st)
{
    return pb.dtype == 0 ? launch_to_dense_t<float>(pb, R, L, M, st) : launch_to_dense_t<bf16_t>(pb, R, L, M, st);
}

// ------------------------------------------------------- bias: add and gradient ----
//
// y[b][o] += bias[o] in place, for the forward kernels that have no bias epilogue of their own; y is
// walked as (row chunk) x (tile of 64 * CW columns) like dy in the column sums (monarch_colsum.h).
template <typename T, int CW>
__global__ void __launch_bounds__(64 * ROWCOL_WAVES)
bias_add_kernel(T* __restrict__ y, const T* __restrict__ bias, int64_t B, int n_out, int col_tiles, int chunks)
{
    const int ct = blockIdx.x % col_tiles, ch = blockIdx.x / col_tiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = (ct * 64 + lane) * CW;
    if (col >= n_out) return;
    const int64_t rows_per = (B + chunks - 1) / chunks;
    const int64_t r0 = ch * rows_per;
    int64_t r1 = r0 + rows_per;
    if (r1 > B) r1 = B;
    float bv[CW];
    ColVec<T, CW>::load(bias + col, bv);
    int64_t r = r0 + wave;
    for (; r + 3 * ROWCOL_WAVES < r1; r += 4 * ROWCOL_WAVES) {
        float v[4][CW];
#pragma unroll
        for (int u = 0; u < 4; ++u) ColVec<T, CW>::load(y + (size_t)(r + u * ROWCOL_WAVES) * n_out + col, v[u]);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < CW; ++e) v[u][e] += bv[e];
            ColVec<T, CW>::store(y + (size_t)(r + u * ROWCOL_WAVES) * n_out + col, v[u]);
        }
    }
    for (; r < r1; r += ROWCOL_WAVES) {
        float v[CW];
        ColVec<T, CW>::load(y + (size_t)r * n_out + col, v);
#pragma unroll
        for (int e = 0; e < CW; ++e) v[e] += bv[e];
        ColVec<T, CW>::store(y + (size_t)r * n_out + col, v);
    }
}

template <typename T>
static void launch_bias_add_t(const Problem& pb, void* y, hipStream_t st)
{
    const int n_out = pb.n_out(), col_tiles = rowcol_col_tiles(n_out), chunks = rowcol_chunks(pb.B, n_out);
    const dim3 grid((unsigned)(col_tiles * chunks)), block(64 * ROWCOL_WAVES);
    if (rowcol_cw(n_out) == 4)
        hipLaunchKernelGGL((bias_add_kernel<T, 4>), grid, block, 0, st, (T*)y, (const T*)pb.bias, pb.B, n_out, col_tiles, chunks);
    else
        hipLaunchKernelGGL((bias_add_kernel<T, 1>), grid, block, 0, st, (T*)y, (const T*)pb.bias, pb.B, n_out, col_tiles, chunks);
}

int launch_bias_add(const Problem& pb, void* y, hipStream_t st)
{
    if (pb.B == 0) return 0;
    if (pb.dtype == 0) launch_bias_add_t<float>(pb, y, st);
    else launch_bias_add_t<bf16_t>(pb, y, st);
    return hip_status(hipGetLastError());
}

// dbias[o] = sum_b dy[b][o] as two kernels of its own (bodies in monarch_colsum.h); the k = 4 matrix-core
// backward runs the same bodies at the tail of two of its own launches instead.
size_t colsum_workspace(const Problem& pb)
{
    return align_up((size_t)rowcol_chunks(pb.B, pb.n_out()) * pb.n_out() * sizeof(float), 256);
}

template <typename T, int CW>
__global__ void __launch_bounds__(64 * ROWCOL_WAVES) colsum_partial_kernel(ColsumJob cj)
{
    colsum_partial_body<T, CW>(cj, (int)blockIdx.x);
}

template <typename TO>
__global__ void __launch_bounds__(1024) colsum_final_kernel(ColsumJob cj)
{
    colsum_final_body<TO, 16>(cj, (int)blockIdx.x);
}

ColsumJob make_colsum_job(const Problem& pb, const void* dy, void* dbias, void* ws)
{
    ColsumJob cj;
    cj.dy = dy;
    cj.part = (float*)ws;
    cj.dbias = dbias;
    cj.B = pb.B;
    cj.n_out = pb.n_out();
    cj.col_tiles = rowcol_col_tiles(cj.n_out);
    cj.chunks = rowcol_chunks(pb.B, cj.n_out);
    cj.out_f32 = pb.wgrad_f32() ? 1 : 0;
    return cj;
}

// ws: colsum_workspace(pb) bytes.  dbias is fp32 when pb.wgrad_f32(), else of pb.dtype.
int launch_colsum(const Problem& pb, const void* dy, void* dbias, void* ws, hipStream_t st)
{
    const int n_out = pb.n_out();
    if (pb.B == 0) {
        if (pb.wgrad_f32()) return launch_fill_zero_f32((float*)dbias, n_out, st);
        return launch_fill_zero_u16((uint16_t*)dbias, n_out, st);
    }
    const ColsumJob cj = make_colsum_job(pb, dy, dbias, ws);
    const dim3 grid((unsigned)colsum_partial_blocks(cj)), block(64 * ROWCOL_WAVES);
    const bool cw4 = rowcol_cw(n_out) == 4;
    if (pb.dtype == 0) {
        if (cw4) hipLaunchKernelGGL((colsum_partial_kernel<float, 4>), grid, block, 0, st, cj);
        else hipLaunchKernelGGL((colsum_partial_kernel<float, 1>), grid, block, 0, st, cj);
    } else {
        if (cw4) hipLaunchKernelGGL((colsum_partial_kernel<bf16_t, 4>), grid, block, 0, st, cj);
        else hipLaunchKernelGGL((colsum_partial_kernel<bf16_t, 1>), grid, block, 0, st, cj);
    }
    if (hipGetLastError() != hipSuccess) return -4;
    const dim3 g2((unsigned)colsum_final_blocks(cj));
    if (cj.out_f32) hipLaunchKernelGGL(colsum_final_kernel<float>, g2, dim3(1024), 0, st, cj);
    else hipLaunchKernelGGL(colsum_final_kernel<bf16_t>, g2, dim3(1024), 0, st, cj);
    return hip_status(hipGetLastError());
}

// -------------------------------------------------------------------- forward ----
//
// LDS: xs[BM][n_in] and us[BM][k*q], both fp32.  Each thread owns one output column at a
// time and keeps BM row accumulators, so every weight is read once per workgroup.

template <typename T, int BM>
__global__ void __launch_bounds__(kThreads)
generic_fwd_kernel(const T* __restrict__ x, const T* __restrict__ R, const T* __restrict__ L,
                   const T* __restrict__ bias, T* __restrict__ y, int64_t B, int k, int p, int q, int s, int perm_b)
{
    extern __shared__ float lds[];
    const int n_in = k * p, kq = k * q, n_out = k * s;
    float* xs = lds;
    float* us = lds + (size_t)BM * n_in;
    const int64_t b0 = (int64_t)blockIdx.x * BM;
    const int tid = threadIdx.x;

    for (int e = tid; e < BM * n_in; e += kThreads) {
        int b = e / n_in, c = e - b * n_in;
        int64_t row = b0 + b;
        xs[e] = row < B ? Elem<T>::load(x + row * n_in + c) : 0.f;
    }
    __syncthreads();

    // step 1 (block-diagonal R) with the mid permutation folded into the LDS store
    for (int f = tid; f < kq; f += kThreads) {
        const int kk = f / q;
        const T* Rrow = R + (size_t)f * p;
        const float* xk = xs + kk * p;
        float acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = 0.f;
        for (int i = 0; i < p; ++i) {
            const float w = Elem<T>::load(Rrow + i);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = fmaf(w, xk[b * n_in + i], acc[b]);
        }
        const int g = mid_dest(f, k, q, perm_b != 0);
#pragma unroll
        for (int b = 0; b < BM; ++b) us[b * kq + g] = acc[b];
    }
    __syncthreads();

    // step 2 (block-diagonal L) and step 3 (output index l*k + c)
    for (int o = tid; o < n_out; o += kThreads) {
        const int l = o / k, c = o - l * k;
        const T* Lrow = L + ((size_t)c * s + l) * q;
        const float* uc = us + c * q;
        float acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = 0.f;
        for (int r = 0; r < q; ++r) {
            const float w = Elem<T>::load(Lrow + r);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = fmaf(w, uc[b * kq + r], acc[b]);
        }
        const float bo = bias ? Elem<T>::load(bias + o) : 0.f;
#pragma unroll
        for (int b = 0; b < BM; ++b) {
            int64_t row = b0 + b;
            if (row < B) Elem<T>::store(y + row * n_out + o, bias ? acc[b] + bo : acc[b]);
        }
    }
}

// ----------------------------------------------------------- transposed multiply ----
//
// y = x M (the rows of x have length k*s, those of y k*p): undo the outer permutation, multiply by the
// transposed blocks of L, undo the mid permutation, multiply by the transposed blocks of R.
// LDS (fp32): ws[BM][k*s] (W[b][c*s + l] = x[b][l*k + c]) and us[BM][k*q] (the vector between the factors).

template <typename T, int BM>
__global__ void __launch_bounds__(kThreads)
generic_fwd_t_kernel(const T* __restrict__ x, const T* __restrict__ R, const T* __restrict__ L, T* __restrict__ y,
                     int64_t B, int k, int p, int q, int s, int perm_b)
{
    extern __shared__ float lds[];
    const int n_in = k * p, kq = k * q, n_out = k * s;
    float* ws = lds;
    float* us = ws + (size_t)BM * n_out;
    const int64_t b0 = (int64_t)blockIdx.x * BM;
    const int tid = threadIdx.x;
    const bool pb = perm_b != 0;

    for (int e = tid; e < BM * n_out; e += kThreads) {
        int b = e / n_out, o = e - b * n_out;
        int l = o / k, c = o - l * k;
        int64_t row = b0 + b;
        ws[b * n_out + c * s + l] = row < B ? Elem<T>::load(x + row * n_out + o) : 0.f;
    }
    __syncthreads();
    // U[c*q + r] = sum_l L[c][l][r] W[c][l]
    for (int g = tid; g < kq; g += kThreads) {
        const int c = g / q, r = g - c * q;
        const T* Lcol = L + (size_t)c * s * q + r;
        const float* wc = ws + c * s;
        float acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = 0.f;
        for (int l = 0; l < s; ++l) {
            const float w = Elem<T>::load(Lcol + (size_t)l * q);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = fmaf(w, wc[b * n_out + l], acc[b]);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) us[b * kq + g] = acc[b];
    }
    __syncthreads();
    // y[kk*p + i] = sum_j R[kk][j][i] U[position that stage-1 output (kk, j) is moved to]
    for (int n = tid; n < n_in; n += kThreads) {
        const int kk = n / p, i = n - kk * p;
        const T* Rcol = R + (size_t)kk * q * p + i;
        float acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = 0.f;
        for (int j = 0; j < q; ++j) {
            const float w = Elem<T>::load(Rcol + (size_t)j * p);
            const int g = mid_dest(kk * q + j, k, q, pb);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = fmaf(w, us[b * kq + g], acc[b]);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) {
            int64_t row = b0 + b;
            if (row < B) Elem<T>::store(y + row * n_in + n, acc[b]);
        }
    }
}

static size_t fwd_t_floats_per_row(const Problem& pb) { return (size_t)pb.n_out() + pb.kq(); }

template <typename T, int BM>
static int launch_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    const size_t lds = (size_t)BM * fwd_t_floats_per_row(pb) * sizeof(float);
    auto kern = generic_fwd_t_kernel<T, BM>;
    hipError_t e = allow_dynamic_lds((const void*)kern, lds);
    if (e != hipSuccess) return -4;
    const int64_t grid = (pb.B + BM - 1) / BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), lds, st, (const T*)x, (const T*)R, (const T*)L,
                       (T*)y, pb.B, pb.k, pb.p, pb.q, pb.s, pb.perm_b() ? 1 : 0);
    return hip_status(hipGetLastError());
}

// ------------------------------------------------------------------- backward ----
//
// LDS (fp32): xs[BM][n_in], us[BM][kq] (U recomputed), dws[BM][k*s] (dW[b][c*s+l]),
// dus[BM][kq] (dU; dY1[f] is read back as dus[mid_dest(f)]).
// dx is written directly; dR and dL contributions of the tile are added with fp32 atomics
// into accumulators that the host zero-filled before the launch.

template <typename T, int BM>
__global__ void __launch_bounds__(kThreads)
generic_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x, const T* __restrict__ R,
                   const T* __restrict__ L, T* __restrict__ dx, float* __restrict__ dRacc,
                   float* __restrict__ dLacc, int64_t B, int k, int p, int q, int s, int perm_b)
{
    extern __shared__ float lds[];
    const int n_in = k * p, kq = k * q, n_out = k * s;
    float* xs = lds;
    float* us = xs + (size_t)BM * n_in;
    float* dws = us + (size_t)BM * kq;
    float* dus = dws + (size_t)BM * n_out;
    const int64_t b0 = (int64_t)blockIdx.x * BM;
    const int tid = threadIdx.x;
    const bool pb = perm_b != 0;

    for (int e = tid; e < BM * n_in; e += kThreads) {
        int b = e / n_in, c = e - b * n_in;
        int64_t row = b0 + b;
        xs[e] = row < B ? Elem<T>::load(x + row * n_in + c) : 0.f;
    }
    for (int e = tid; e < BM * n_out; e += kThreads) {
        int b = e / n_out, o = e - b * n_out;
        int l = o / k, c = o - l * k;
        int64_t row = b0 + b;
        dws[b * n_out + c * s + l] = row < B ? Elem<T>::load(dy + row * n_out + o) : 0.f;
    }
    __syncthreads();

    // recompute step 1 + mid permutation
    for (int f = tid; f < kq; f += kThreads) {
        const int kk = f / q;
        const T* Rrow = R + (size_t)f * p;
        const float* xk = xs + kk * p;
        float acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = 0.f;
        for (int i = 0; i < p; ++i) {
            const float w = Elem<T>::load(Rrow + i);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = fmaf(w, xk[b * n_in + i], acc[b]);
        }
        const int g = mid_dest(f, k, q, pb);
#pragma unroll
        for (int b = 0; b < BM; ++b) us[b * kq + g] = acc[b];
    }
    // adjoint of step 2: dU[c*q + r] = sum_l L[c][l][r] dW[c][l]
    for (int g = tid; g < kq; g += kThreads) {
        const int c = g / q, r = g - c * q;
        const T* Lcol = L + (size_t)c * s * q + r;
        const float* dwc = dws + c * s;
        float acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = 0.f;
        for (int l = 0; l < s; ++l) {
            const float w = Elem<T>::load(Lcol + (size_t)l * q);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = fmaf(w, dwc[b * n_out + l], acc[b]);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) dus[b * kq + g] = acc[b];
    }
    __syncthreads();

    // adjoint of step 1, data part: dx[kk*p + i] = sum_j R[kk][j][i] dY1[kk][j]
    for (int n = tid; n < n_in; n += kThreads) {
        const int kk = n / p, i = n - kk * p;
        const T* Rcol = R + (size_t)kk * q * p + i;
        float acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = 0.f;
        for (int j = 0; j < q; ++j) {
            const float w = Elem<T>::load(Rcol + (size_t)j * p);
            const int g = mid_dest(kk * q + j, k, q, pb);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = fmaf(w, dus[b * kq + g], acc[b]);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) {
            int64_t row = b0 + b;
            if (row < B) Elem<T>::store(dx + row * n_in + n, acc[b]);
        }
    }
    // weight gradients of this tile (rows beyond B contribute zeros)
    const int nL = k * s * q;
    for (int e = tid; e < nL; e += kThreads) {
        const int cl = e / q, r = e - cl * q;
        const int c = cl / s;
        float v = 0.f;
#pragma unroll
        for (int b = 0; b < BM; ++b) v = fmaf(dws[b * n_out + cl], us[b * kq + c * q + r], v);
        unsafeAtomicAdd(dLacc + e, v);
    }
    const int nR = kq * p;
    for (int e = tid; e < nR; e += kThreads) {
        const int f = e / p, i = e - f * p;
        const int kk = f / q;
        const int g = mid_dest(f, k, q, pb);
        float v = 0.f;
#pragma unroll
        for (int b = 0; b < BM; ++b) v = fmaf(dus[b * kq + g], xs[b * n_in + kk * p + i], v);
        unsafeAtomicAdd(dRacc + e, v);
    }
}

// ------------------------------------------------------------------ launchers ----

static int pick_bm(size_t floats_per_row)
{
    for (int bm = 8; bm >= 1; bm >>= 1)
        if ((size_t)bm * floats_per_row * sizeof(float) <= kMaxLdsBytes) return bm;
    return 0;
}

static size_t fwd_floats_per_row(const Problem& pb) { return (size_t)pb.n_in + pb.kq(); }
static size_t bwd_floats_per_row(const Problem& pb)
{
    return (size_t)pb.n_in + 2 * (size_t)pb.kq() + pb.n_out();
}

bool generic_fwd_supported(const Problem& pb) { return pick_bm(fwd_floats_per_row(pb)) > 0; }
bool generic_bwd_supported(const Problem& pb) { return pick_bm(bwd_floats_per_row(pb)) > 0; }

size_t generic_bwd_workspace(const Problem& pb)
{
    if (pb.wgrad_f32()) return 0;  // atomics go straight into dR / dL
    return align_up(pb.n_R() * sizeof(float), 256) + align_up(pb.n_L() * sizeof(float), 256);
}

template <typename T, int BM>
static int launch_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y,
                      hipStream_t st)
{
    const size_t lds = (size_t)BM * fwd_floats_per_row(pb) * sizeof(float);
    auto kern = generic_fwd_kernel<T, BM>;
    hipError_t e = allow_dynamic_lds((const void*)kern, lds);
    if (e != hipSuccess) return -4;
    const int64_t grid = (pb.B + BM - 1) / BM;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), lds, st, (const T*)x, (const T*)R,
                       (const T*)L, (const T*)pb.bias, (T*)y, pb.B, pb.k, pb.p, pb.q, pb.s, pb.perm_b() ? 1 : 0);
    return hip_status(hipGetLastError());
}

template <typename T>
static int dispatch_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y,
                        hipStream_t st)
{
    switch (pick_bm(fwd_floats_per_row(pb))) {
        case 8: return launch_fwd<T, 8>(pb, x, R, L, y, st);
        case 4: return launch_fwd<T, 4>(pb, x, R, L, y, st);
        case 2: return launch_fwd<T, 2>(pb, x, R, L, y, st);
        case 1: return launch_fwd<T, 1>(pb, x, R, L, y, st);
        default: return -2;
    }
}

int generic_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    if ((pb.B + 7) / 8 > 0x7fffffffLL) return -2;
    return pb.dtype == 0 ? dispatch_fwd<float>(pb, x, R, L, y, st)
                         : dispatch_fwd<bf16_t>(pb, x, R, L, y, st);
}

template <typename T, int BM>
static int launch_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L,
                      void* dx, float* dRacc, float* dLacc, hipStream_t st)
{
    const size_t lds = (size_t)BM * bwd_floats_per_row(pb) * sizeof(float);
    auto kern = generic_bwd_kernel<T, BM>;
    hipError_t e = allow_dynamic_lds((const void*)kern, lds);
    if (e != hipSuccess) return -4;
    const int64_t grid = (pb.B + BM - 1) / BM;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kThreads), lds, st, (const T*)dy, (const T*)x,
                       (const T*)R, (const T*)L, (T*)dx, dRacc, dLacc, pb.B, pb.k, pb.p, pb.q, pb.s,
                       pb.perm_b() ? 1 : 0);
    return hip_status(hipGetLastError());
}

template <typename T>
static int dispatch_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L,
                        void* dx, float* dRacc, float* dLacc, hipStream_t st)
{
    switch (pick_bm(bwd_floats_per_row(pb))) {
        case 8: return launch_bwd<T, 8>(pb, dy, x, R, L, dx, dRacc, dLacc, st);
        case 4: return launch_bwd<T, 4>(pb, dy, x, R, L, dx, dRacc, dLacc, st);
        case 2: return launch_bwd<T, 2>(pb, dy, x, R, L, dx, dRacc, dLacc, st);
        case 1: return launch_bwd<T, 1>(pb, dy, x, R, L, dx, dRacc, dLacc, st);
        default: return -2;
    }
}

int generic_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L,
                void* dx, void* dR, void* dL, void* ws, hipStream_t st)
{
    if ((pb.B + 7) / 8 > 0x7fffffffLL) return -2;
    float* dRacc;
    float* dLacc;
    if (pb.wgrad_f32()) {
        dRacc = (float*)dR;
        dLacc = (float*)dL;
    } else {
        dRacc = (float*)ws;
        dLacc = (float*)((char*)ws + align_up(pb.n_R() * sizeof(float), 256));
    }
    int rc = launch_fill_zero_f32(dRacc, pb.n_R(), st);
    if (rc) return rc;
    rc = launch_fill_zero_f32(dLacc, pb.n_L(), st);
    if (rc) return rc;
    if (pb.B > 0) {
        rc = pb.dtype == 0 ? dispatch_bwd<float>(pb, dy, x, R, L, dx, dRacc, dLacc, st)
                           : dispatch_bwd<bf16_t>(pb, dy, x, R, L, dx, dRacc, dLacc, st);
        if (rc) return rc;
    }
    if (!pb.wgrad_f32()) {
        rc = launch_f32_to_bf16(dRacc, (uint16_t*)dR, pb.n_R(), st);
        if (rc) return rc;
        rc = launch_f32_to_bf16(dLacc, (uint16_t*)dL, pb.n_L(), st);
        if (rc) return rc;
    }
    return 0;
}

bool generic_fwd_t_supported(const Problem& pb)
{
    for (int bm = 8; bm >= 1; bm >>= 1)
        if ((size_t)bm * fwd_t_floats_per_row(pb) * sizeof(float) <= kMaxLdsBytes) return true;
    return false;
}

template <typename T>
static int generic_fwd_t_typed(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    const size_t per_row = fwd_t_floats_per_row(pb) * sizeof(float);
    if (8 * per_row <= kMaxLdsBytes) return launch_fwd_t<T, 8>(pb, x, R, L, y, st);
    if (4 * per_row <= kMaxLdsBytes) return launch_fwd_t<T, 4>(pb, x, R, L, y, st);
    if (2 * per_row <= kMaxLdsBytes) return launch_fwd_t<T, 2>(pb, x, R, L, y, st);
    if (per_row <= kMaxLdsBytes) return launch_fwd_t<T, 1>(pb, x, R, L, y, st);
    return -2;
}

int generic_fwd_t(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    return pb.dtype == 0 ? generic_fwd_t_typed<float>(pb, x, R, L, y, st) : generic_fwd_t_typed<bf16_t>(pb, x, R, L, y, st);
}

}  // namespace monarch
