// Complex-valued Monarch multiply (complex64: interleaved fp32 real and imaginary parts) and the
// factors that make the Monarch matrix a DFT.  The paper's results hold over C as well (Notation
// Review), and its MRI model is one complex Monarch matrix initialised to the inverse FFT.
//
// Same steps as the real kernels (Section 3.3 steps 1-3, permutations of Definition 3.1), in the
// shape-generic SIMT form: one workgroup per tile of BM batch rows, the vector between the two factors in
// LDS, one thread per output element with BM complex accumulators, so every weight is read once per
// workgroup.  No transposes are conjugated in the forward (M^T, not M^*).  Gradients use the
// convention of automatic differentiation for a real loss: grad z = dLoss/dRe z + i dLoss/dIm z, i.e.
//   dU = dW conj(L),  dL = dW^T conj(U),  dx = dY1 conj(R),  dR = dY1^T conj(x).
#include "monarch_internal.h"
#include "monarch_device.h"

namespace monarch {
namespace {

constexpr int kCThreads = 256;

struct cf {
    float re, im;
};
__device__ __forceinline__ cf cmul_acc(cf acc, cf a, cf b)  // acc + a * b
{
    acc.re = fmaf(a.re, b.re, fmaf(-a.im, b.im, acc.re));
    acc.im = fmaf(a.re, b.im, fmaf(a.im, b.re, acc.im));
    return acc;
}
__device__ __forceinline__ cf cmul_conj_acc(cf acc, cf a, cf b)  // acc + a * conj(b)
{
    acc.re = fmaf(a.re, b.re, fmaf(a.im, b.im, acc.re));
    acc.im = fmaf(a.im, b.re, fmaf(-a.re, b.im, acc.im));
    return acc;
}
__device__ __forceinline__ cf ldc(const float2* p) { const float2 v = *p; return cf{v.x, v.y}; }

// Only the vector between the two factors is kept in LDS (BM rows of k*q values): the inputs of a stage are read
// from global memory where all lanes of a wave that work on one block ask for the same address (one broadcast load),
// which leaves room for four rows per workgroup at n = 4096 and so a quarter of the weight traffic per row.
// Rows past the end of the batch are computed from the last row and not stored.
template <int BM>
__global__ void __launch_bounds__(kCThreads)
complex_fwd_kernel(const float2* __restrict__ x, const float2* __restrict__ R, const float2* __restrict__ L,
                   float2* __restrict__ y, int64_t B, int k, int p, int q, int s, int perm_b)
{
    extern __shared__ float2 ldsc[];
    const int n_in = k * p, kq = k * q, n_out = k * s;
    float2* us = ldsc;
    const int64_t b0 = (int64_t)blockIdx.x * BM;
    const int tid = threadIdx.x;
    const float2* xrow[BM];
#pragma unroll
    for (int b = 0; b < BM; ++b) xrow[b] = x + (b0 + b < B ? b0 + b : B - 1) * n_in;
    for (int f = tid; f < kq; f += kCThreads) {
        const int kk = f / q;
        const float2* Rrow = R + (size_t)f * p;
        cf acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = cf{0.f, 0.f};
        for (int i = 0; i < p; ++i) {
            const cf w = ldc(Rrow + i);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = cmul_acc(acc[b], w, ldc(xrow[b] + kk * p + i));
        }
        const int g = mid_dest(f, k, q, perm_b != 0);
#pragma unroll
        for (int b = 0; b < BM; ++b) us[b * kq + g] = make_float2(acc[b].re, acc[b].im);
    }
    __syncthreads();
    for (int o = tid; o < n_out; o += kCThreads) {
        const int l = o / k, c = o - l * k;
        const float2* Lrow = L + ((size_t)c * s + l) * q;
        const float2* uc = us + c * q;
        cf acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = cf{0.f, 0.f};
        for (int r = 0; r < q; ++r) {
            const cf w = ldc(Lrow + r);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = cmul_acc(acc[b], w, ldc(uc + b * kq + r));
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) {
            const int64_t row = b0 + b;
            if (row < B) y[row * n_out + o] = make_float2(acc[b].re, acc[b].im);
        }
    }
}

// LDS: us[BM][kq] (U recomputed) and dus[BM][kq] (dU); x and dy are read from global memory (see above).
// dx is written directly.  WS = false: the dR and dL contributions of the tile are added with fp32 atomics (one per
// component) into dR / dL, which the host zero-filled before the launch.  WS = true: the three batch-major operands of
// the weight gradients go to the workspace instead -- U[b][c*q + r], dY1[b][kk*q + j] (mid permutation undone) and
// dW[b][c*s + l] (outer permutation undone) -- and complex_wgrad_kernel contracts them over the batch.
template <int BM, bool WS>
__global__ void __launch_bounds__(kCThreads)
complex_bwd_kernel(const float2* __restrict__ dy, const float2* __restrict__ x, const float2* __restrict__ R,
                   const float2* __restrict__ L, float2* __restrict__ dx, float* __restrict__ dRacc,
                   float* __restrict__ dLacc, float2* __restrict__ Uws, float2* __restrict__ dY1ws,
                   float2* __restrict__ dWws, int64_t B, int k, int p, int q, int s, int perm_b)
{
    extern __shared__ float2 ldsc[];
    const int n_in = k * p, kq = k * q, n_out = k * s;
    float2* us = ldsc;
    float2* dus = us + (size_t)BM * kq;
    const int64_t b0 = (int64_t)blockIdx.x * BM;
    const int tid = threadIdx.x;
    const bool pb = perm_b != 0;
    const float2* xrow[BM];
    const float2* dyrow[BM];
#pragma unroll
    for (int b = 0; b < BM; ++b) {
        const int64_t row = b0 + b < B ? b0 + b : B - 1;
        xrow[b] = x + row * n_in;
        dyrow[b] = dy + row * n_out;
    }
    for (int f = tid; f < kq; f += kCThreads) {  // step 1 again, with the mid permutation
        const int kk = f / q;
        const float2* Rrow = R + (size_t)f * p;
        cf acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = cf{0.f, 0.f};
        for (int i = 0; i < p; ++i) {
            const cf w = ldc(Rrow + i);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = cmul_acc(acc[b], w, ldc(xrow[b] + kk * p + i));
        }
        const int g = mid_dest(f, k, q, pb);
#pragma unroll
        for (int b = 0; b < BM; ++b) us[b * kq + g] = make_float2(acc[b].re, acc[b].im);
    }
    for (int g = tid; g < kq; g += kCThreads) {  // dU[c*q + r] = sum_l dW[c][l] conj(L[c][l][r]),  dW[c][l] = dy[l*k + c]
        const int c = g / q, r = g - c * q;
        const float2* Lcol = L + (size_t)c * s * q + r;
        cf acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = cf{0.f, 0.f};
        for (int l = 0; l < s; ++l) {
            const cf w = ldc(Lcol + (size_t)l * q);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = cmul_conj_acc(acc[b], ldc(dyrow[b] + (size_t)l * k + c), w);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) dus[b * kq + g] = make_float2(acc[b].re, acc[b].im);
    }
    __syncthreads();
    for (int n = tid; n < n_in; n += kCThreads) {  // dx[kk*p + i] = sum_j dY1[kk][j] conj(R[kk][j][i])
        const int kk = n / p, i = n - kk * p;
        const float2* Rcol = R + (size_t)kk * q * p + i;
        cf acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = cf{0.f, 0.f};
        for (int j = 0; j < q; ++j) {
            const cf w = ldc(Rcol + (size_t)j * p);
            const int g = mid_dest(kk * q + j, k, q, pb);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = cmul_conj_acc(acc[b], ldc(dus + b * kq + g), w);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) {
            const int64_t row = b0 + b;
            if (row < B) dx[row * n_in + n] = make_float2(acc[b].re, acc[b].im);
        }
    }
    if constexpr (WS) {
        for (int e = tid; e < BM * kq; e += kCThreads) {
            const int b = e / kq, f = e - b * kq;
            const int64_t row = b0 + b;
            if (row < B) {
                Uws[row * kq + f] = us[e];
                dY1ws[row * kq + f] = dus[b * kq + mid_dest(f, k, q, pb)];
            }
        }
        for (int e = tid; e < BM * n_out; e += kCThreads) {
            const int b = e / n_out, cl = e - b * n_out;
            const int c = cl / s, l = cl - c * s;
            const int64_t row = b0 + b;
            if (row < B) dWws[row * n_out + cl] = dy[row * n_out + (size_t)l * k + c];
        }
        return;
    }
    const int nL = k * s * q;
    for (int e = tid; e < nL; e += kCThreads) {  // dL[c][l][r] += sum_b dW[b][c][l] conj(U[b][c][r])
        const int cl = e / q, r = e - cl * q;
        const int c = cl / s, l = cl - c * s;
        cf v = cf{0.f, 0.f};
#pragma unroll
        for (int b = 0; b < BM; ++b)
            if (b0 + b < B) v = cmul_conj_acc(v, ldc(dyrow[b] + (size_t)l * k + c), ldc(us + b * kq + c * q + r));
        unsafeAtomicAdd(dLacc + 2 * (size_t)e, v.re);
        unsafeAtomicAdd(dLacc + 2 * (size_t)e + 1, v.im);
    }
    const int nR = kq * p;
    for (int e = tid; e < nR; e += kCThreads) {  // dR[kk][j][i] += sum_b dY1[b][kk][j] conj(x[b][kk*p + i])
        const int f = e / p, i = e - f * p;
        const int kk = f / q;
        const int g = mid_dest(f, k, q, pb);
        cf v = cf{0.f, 0.f};
#pragma unroll
        for (int b = 0; b < BM; ++b)
            if (b0 + b < B) v = cmul_conj_acc(v, ldc(dus + b * kq + g), ldc(xrow[b] + kk * p + i));
        unsafeAtomicAdd(dRacc + 2 * (size_t)e, v.re);
        unsafeAtomicAdd(dRacc + 2 * (size_t)e + 1, v.im);
    }
}

// out[g][m][n] += sum over the rows b of batch chunk blockIdx.y of  A[b][g*a_g + m] * conj(Bm[b][g*b_g + n])
// (complex64, fp32 arithmetic): both weight gradients of the complex backward, dL[c] = dW[c]^T conj(U[c]) and
// dR[kk] = dY1[kk]^T conj(x[kk]), in one launch.  A workgroup owns a 64 x 64 tile of one group: 16 x 16 threads with
// 4 x 4 accumulators each, the operands of 16 batch rows at a time staged in LDS; entries beyond M, N or the batch
// read as zeros.  The chunks' partial tiles are added with fp32 atomics into the zero-filled outputs.
struct CGemm {
    const float2* A;
    int64_t lda;
    int a_g;
    const float2* Bm;
    int64_t ldb;
    int b_g;
    int M, N, G;
    float* out;
};
constexpr int kCT = 64, kCK = 16;

__global__ void __launch_bounds__(256)
complex_wgrad_kernel(CGemm d0, CGemm d1, int tiles0, int64_t rows, int64_t rows_per_chunk)
{
    __shared__ float2 As[kCK][kCT + 1], Bs[kCK][kCT + 1];
    const bool first = (int)blockIdx.x < tiles0;
    const CGemm& d = first ? d0 : d1;
    int t = (int)blockIdx.x - (first ? 0 : tiles0);
    const int tn_count = (d.N + kCT - 1) / kCT, tm_count = (d.M + kCT - 1) / kCT;
    const int tn = t % tn_count; t /= tn_count;
    const int tm = t % tm_count;
    const int g = t / tm_count;
    const int m0 = tm * kCT, n0 = tn * kCT;
    const int64_t row_lo = (int64_t)blockIdx.y * rows_per_chunk;
    const int64_t row_hi = row_lo + rows_per_chunk < rows ? row_lo + rows_per_chunk : rows;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    cf acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = cf{0.f, 0.f};
    const float2 zero = make_float2(0.f, 0.f);
    for (int64_t r0 = row_lo; r0 < row_hi; r0 += kCK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + i * 256;
            const int rr = idx / kCT, cc = idx % kCT;
            const int64_t row = r0 + rr;
            As[rr][cc] = (row < row_hi && m0 + cc < d.M) ? d.A[row * d.lda + (size_t)g * d.a_g + m0 + cc] : zero;
            Bs[rr][cc] = (row < row_hi && n0 + cc < d.N) ? d.Bm[row * d.ldb + (size_t)g * d.b_g + n0 + cc] : zero;
        }
        __syncthreads();
#pragma unroll
        for (int kb = 0; kb < kCK; ++kb) {
            cf a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = ldc(&As[kb][ty * 4 + i]);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = ldc(&Bs[kb][tx * 4 + j]);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = cmul_conj_acc(acc[i][j], a[i], b[j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < d.M && n < d.N) {
                float* o = d.out + 2 * (((size_t)g * d.M + m) * d.N + n);
                unsafeAtomicAdd(o, acc[i][j].re);
                unsafeAtomicAdd(o + 1, acc[i][j].im);
            }
        }
}

// y = x conj(M): the conjugate transpose M* applied to every row (the second factor of a product M1 M2* of
// Section 3.1), i.e. the two dx stages of the kernel above on their own: x (B, k*s) -> y (B, k*p).
// LDS: dus[BM][kq].
template <int BM>
__global__ void __launch_bounds__(kCThreads)
complex_fwd_h_kernel(const float2* __restrict__ x, const float2* __restrict__ R, const float2* __restrict__ L,
                     float2* __restrict__ y, int64_t B, int k, int p, int q, int s, int perm_b)
{
    extern __shared__ float2 ldsc[];
    const int n_in = k * p, kq = k * q, n_out = k * s;
    float2* dus = ldsc;
    const int64_t b0 = (int64_t)blockIdx.x * BM;
    const int tid = threadIdx.x;
    const bool pb = perm_b != 0;
    const float2* xrow[BM];
#pragma unroll
    for (int b = 0; b < BM; ++b) xrow[b] = x + (b0 + b < B ? b0 + b : B - 1) * n_out;
    for (int g = tid; g < kq; g += kCThreads) {  // V[c*q + r] = sum_l W[c][l] conj(L[c][l][r]),  W[c][l] = x[l*k + c]
        const int c = g / q, r = g - c * q;
        const float2* Lcol = L + (size_t)c * s * q + r;
        cf acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = cf{0.f, 0.f};
        for (int l = 0; l < s; ++l) {
            const cf w = ldc(Lcol + (size_t)l * q);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = cmul_conj_acc(acc[b], ldc(xrow[b] + (size_t)l * k + c), w);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) dus[b * kq + g] = make_float2(acc[b].re, acc[b].im);
    }
    __syncthreads();
    for (int n = tid; n < n_in; n += kCThreads) {  // y[kk*p + i] = sum_j T[kk][j] conj(R[kk][j][i])
        const int kk = n / p, i = n - kk * p;
        const float2* Rcol = R + (size_t)kk * q * p + i;
        cf acc[BM];
#pragma unroll
        for (int b = 0; b < BM; ++b) acc[b] = cf{0.f, 0.f};
        for (int j = 0; j < q; ++j) {
            const cf w = ldc(Rcol + (size_t)j * p);
            const int g = mid_dest(kk * q + j, k, q, pb);
#pragma unroll
            for (int b = 0; b < BM; ++b) acc[b] = cmul_conj_acc(acc[b], ldc(dus + b * kq + g), w);
        }
#pragma unroll
        for (int b = 0; b < BM; ++b) {
            const int64_t row = b0 + b;
            if (row < B) y[row * n_in + n] = make_float2(acc[b].re, acc[b].im);
        }
    }
}

// R[kk][j][i] = w^(i*j*m),  L[j][l][kk] = w^(kk*j + kk*l*m) (times 1/n for the inverse),  w = exp(-+2 pi i / n):
// the 4-step splitting of the DFT of the grid-transposed input, P L P^T R = F_n P.  Exponents are reduced
// mod n in integers and the sine / cosine taken in double precision, then rounded to fp32.
__global__ void __launch_bounds__(256) dft_factors_kernel(float2* __restrict__ R, float2* __restrict__ L, int m, int inverse)
{
    const int n = m * m;
    const int64_t total = (int64_t)m * m * m;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int a = (int)(e / n), b = (int)((e / m) % m), c = (int)(e % m);
    const double sgn = inverse ? 2.0 : -2.0;
    {  // R[kk = a][j = b][i = c]
        const int64_t ex = ((int64_t)c * b * m) % n;
        double sn, cs;
        sincospi(sgn * (double)ex / (double)n, &sn, &cs);
        R[e] = make_float2((float)cs, (float)sn);
    }
    {  // L[j = a][l = b][kk = c]
        const int64_t ex = ((int64_t)c * a + (int64_t)c * b * m) % n;
        double sn, cs;
        sincospi(sgn * (double)ex / (double)n, &sn, &cs);
        const double scale = inverse ? 1.0 / (double)n : 1.0;
        L[e] = make_float2((float)(cs * scale), (float)(sn * scale));
    }
}

size_t fwd_bytes_per_row(const Problem& pb) { return (size_t)pb.kq() * sizeof(float2); }
size_t fwd_h_bytes_per_row(const Problem& pb) { return (size_t)pb.kq() * sizeof(float2); }
size_t bwd_bytes_per_row(const Problem& pb) { return 2 * (size_t)pb.kq() * sizeof(float2); }

int pick_rows(size_t bytes_per_row)
{
    for (int bm = 4; bm >= 1; bm >>= 1)
        if ((size_t)bm * bytes_per_row <= kMaxLdsBytes) return bm;
    return 0;
}

template <int BM>
int launch_cfwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    const size_t lds = (size_t)BM * fwd_bytes_per_row(pb);
    auto kern = complex_fwd_kernel<BM>;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    const int64_t grid = (pb.B + BM - 1) / BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kCThreads), lds, st, (const float2*)x, (const float2*)R,
                       (const float2*)L, (float2*)y, pb.B, pb.k, pb.p, pb.q, pb.s, pb.perm_b() ? 1 : 0);
    return hip_status(hipGetLastError());
}

template <int BM>
int launch_cfwd_h(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    const size_t lds = (size_t)BM * fwd_h_bytes_per_row(pb);
    auto kern = complex_fwd_h_kernel<BM>;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    const int64_t grid = (pb.B + BM - 1) / BM;
    if (grid > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kCThreads), lds, st, (const float2*)x, (const float2*)R,
                       (const float2*)L, (float2*)y, pb.B, pb.k, pb.p, pb.q, pb.s, pb.perm_b() ? 1 : 0);
    return hip_status(hipGetLastError());
}

// ws == nullptr: weight gradients by atomics from the data kernel; else: operands to the workspace, then the GEMM
template <int BM>
int launch_cbwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                void* dL, void* ws, hipStream_t st)
{
    const size_t lds = (size_t)BM * bwd_bytes_per_row(pb);
    auto kern = ws ? complex_bwd_kernel<BM, true> : complex_bwd_kernel<BM, false>;
    if (allow_dynamic_lds((const void*)kern, lds) != hipSuccess) return -4;
    const int64_t grid = (pb.B + BM - 1) / BM;
    if (grid > 0x7fffffffLL) return -2;
    const size_t act = align_up((size_t)pb.B * pb.kq() * sizeof(float2), 256);
    float2* Uws = (float2*)ws;
    float2* dY1ws = ws ? (float2*)((char*)ws + act) : nullptr;
    float2* dWws = ws ? (float2*)((char*)ws + 2 * act) : nullptr;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kCThreads), lds, st, (const float2*)dy, (const float2*)x,
                       (const float2*)R, (const float2*)L, (float2*)dx, (float*)dR, (float*)dL, Uws, dY1ws, dWws, pb.B,
                       pb.k, pb.p, pb.q, pb.s, pb.perm_b() ? 1 : 0);
    int rc = hip_status(hipGetLastError());
    if (rc || !ws) return rc;
    CGemm gl{dWws, pb.n_out(), pb.s, Uws, pb.kq(), pb.q, pb.s, pb.q, pb.k, (float*)dL};
    CGemm gr{dY1ws, pb.kq(), pb.q, (const float2*)x, pb.n_in, pb.p, pb.q, pb.p, pb.k, (float*)dR};
    auto tiles = [](const CGemm& d) { return (int64_t)d.G * ((d.M + kCT - 1) / kCT) * ((d.N + kCT - 1) / kCT); };
    const int64_t t0 = tiles(gl), t1 = tiles(gr);
    int64_t nz = 1024 / (t0 + t1);  // about four workgroups per CU
    const int64_t maxz = (pb.B + 63) / 64;
    if (nz > maxz) nz = maxz;
    if (nz < 1) nz = 1;
    if (nz > 65535) nz = 65535;
    const int64_t rpc = ((pb.B + nz - 1) / nz + kCK - 1) / kCK * kCK;
    nz = (pb.B + rpc - 1) / rpc;
    if (t0 + t1 > 0x7fffffffLL) return -2;
    hipLaunchKernelGGL(complex_wgrad_kernel, dim3((unsigned)(t0 + t1), (unsigned)nz), dim3(256), 0, st, gl, gr, (int)t0,
                       pb.B, rpc);
    return hip_status(hipGetLastError());
}

}  // namespace

bool complex_fwd_supported(const Problem& pb) { return pick_rows(fwd_bytes_per_row(pb)) > 0; }
bool complex_bwd_supported(const Problem& pb) { return pick_rows(bwd_bytes_per_row(pb)) > 0; }
bool complex_fwd_h_supported(const Problem& pb) { return pick_rows(fwd_h_bytes_per_row(pb)) > 0; }

int complex_fwd_h(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    switch (pick_rows(fwd_h_bytes_per_row(pb))) {
        case 4: return launch_cfwd_h<4>(pb, x, R, L, y, st);
        case 2: return launch_cfwd_h<2>(pb, x, R, L, y, st);
        case 1: return launch_cfwd_h<1>(pb, x, R, L, y, st);
        default: return -2;
    }
}

int complex_fwd(const Problem& pb, const void* x, const void* R, const void* L, void* y, hipStream_t st)
{
    switch (pick_rows(fwd_bytes_per_row(pb))) {
        case 4: return launch_cfwd<4>(pb, x, R, L, y, st);
        case 2: return launch_cfwd<2>(pb, x, R, L, y, st);
        case 1: return launch_cfwd<1>(pb, x, R, L, y, st);
        default: return -2;
    }
}

size_t complex_bwd_workspace(const Problem& pb)
{
    const size_t rows = pb.B > 0 ? (size_t)pb.B : 1;
    return 2 * align_up(rows * pb.kq() * sizeof(float2), 256) + align_up(rows * pb.n_out() * sizeof(float2), 256);
}

int complex_bwd(const Problem& pb, const void* dy, const void* x, const void* R, const void* L, void* dx, void* dR,
                void* dL, void* ws, hipStream_t st)
{
    int rc = launch_fill_zero_f32((float*)dR, 2 * pb.n_R(), st);
    if (rc) return rc;
    rc = launch_fill_zero_f32((float*)dL, 2 * pb.n_L(), st);
    if (rc || pb.B == 0) return rc;
    switch (pick_rows(bwd_bytes_per_row(pb))) {
        case 4: return launch_cbwd<4>(pb, dy, x, R, L, dx, dR, dL, ws, st);
        case 2: return launch_cbwd<2>(pb, dy, x, R, L, dx, dR, dL, ws, st);
        case 1: return launch_cbwd<1>(pb, dy, x, R, L, dx, dR, dL, ws, st);
        default: return -2;
    }
}

int launch_dft_factors(void* R, void* L, int m, int inverse, hipStream_t st)
{
    const int64_t total = (int64_t)m * m * m;
    hipLaunchKernelGGL(dft_factors_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (float2*)R, (float2*)L, m, inverse);
    return hip_status(hipGetLastError());
}

}  // namespace monarch
