// Projection of a dense n x n matrix, n = m^2, onto the square Monarch matrices (Section 3.3,
// Theorem 1, Algorithm 1): with At[l][j][k][i] = A[l*m + j][k*m + i], the slice At[:, j, k, :] of the
// closest Monarch matrix is the best rank-1 approximation sigma_1 u_1 v_1^T of that slice of A, and
// L[j][:][k] = sqrt(sigma_1) u_1,  R[k][j][:] = sqrt(sigma_1) v_1.
//
// The leading singular triple comes from a one-sided (Hestenes) Jacobi SVD, one wavefront per slice:
// lane c owns column c of the slice G (m values in registers) and column c of the accumulated
// rotations V (starts as the identity).  A sweep visits every pair of columns once, m/2 disjoint pairs
// at a time in round-robin tournament order; a pair (p, q) is rotated so that its two columns of G
// become orthogonal, and the same rotation is applied to V, so that G = (slice) * V throughout.  At
// convergence the columns of G are sigma_c u_c and the columns of V are v_c.  Partner columns are read
// with cross-lane shuffles; both lanes of a pair compute the rotation from the same three numbers
// (their squared norms and their inner product, summed in the same order), so they agree bit for bit.
// The sweep loop is bounded (kMaxSweeps), so every wave ends whatever the data.
#include "monarch_internal.h"
#include "monarch_device.h"

namespace monarch {
namespace {

constexpr int kMaxSweeps = 40;
constexpr float kOrthTol = 3e-7f;  // a pair counts as orthogonal when |<p, q>| <= kOrthTol * |p| |q|

template <typename T, int MT>
__global__ void __launch_bounds__(64) project_kernel(const T* __restrict__ A, T* __restrict__ R, T* __restrict__ L, int m)
{
    const int j = blockIdx.x / m, k = blockIdx.x - j * m;
    const int c = threadIdx.x;
    const size_t n = (size_t)m * m;
    float g[MT], v[MT];
#pragma unroll
    for (int r = 0; r < MT; ++r) {
        g[r] = (r < m && c < m) ? Elem<T>::load(A + ((size_t)r * m + j) * n + (size_t)k * m + c) : 0.f;
        v[r] = (r == c && c < m) ? 1.f : 0.f;
    }
    const int me = (m + 1) & ~1;  // players of the tournament: the columns, plus a zero column when m is odd
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        float worst = 0.f;  // largest |<p, q>| / (|p| |q|) met in this sweep
        for (int t = 0; t < me - 1; ++t) {
            int partner = c;
            if (c < me) {
                if (c == me - 1) partner = t;
                else if (c == t) partner = me - 1;
                else {
                    partner = (2 * t - c) % (me - 1);
                    if (partner < 0) partner += me - 1;
                }
            }
            float alpha = 0.f, gamma = 0.f;
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                const float o = __shfl(g[r], partner);
                alpha = fmaf(g[r], g[r], alpha);
                gamma = fmaf(g[r], o, gamma);
            }
            const float beta = __shfl(alpha, partner);
            const bool first = c < partner;
            const float ap = first ? alpha : beta, aq = first ? beta : alpha;
            const float denom = sqrtf(ap) * sqrtf(aq);
            float cs = 1.f, sn = 0.f;
            if (partner != c && fabsf(gamma) > kOrthTol * denom) {
                const float zeta = (aq - ap) / (2.f * gamma);
                const float tt = copysignf(1.f, zeta) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta));
                cs = 1.f / sqrtf(1.f + tt * tt);
                sn = cs * tt;
                worst = fmaxf(worst, fabsf(gamma) / denom);
            }
            // p' = cs p - sn q,  q' = sn p + cs q
            const float mine = cs, theirs = first ? -sn : sn;
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                const float og = __shfl(g[r], partner), ov = __shfl(v[r], partner);
                g[r] = fmaf(theirs, og, mine * g[r]);
                v[r] = fmaf(theirs, ov, mine * v[r]);
            }
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) worst = fmaxf(worst, __shfl_xor(worst, d));
        if (worst == 0.f) break;  // no pair was rotated: every pair is orthogonal to tolerance
    }
    // the column with the largest norm is sigma_1 u_1 (ties: the lowest column index)
    float best = 0.f;
#pragma unroll
    for (int r = 0; r < MT; ++r) best = fmaf(g[r], g[r], best);
    int who = c;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float ob = __shfl_xor(best, d);
        const int ow = __shfl_xor(who, d);
        if (ob > best || (ob == best && ow < who)) {
            best = ob;
            who = ow;
        }
    }
    const float sigma = sqrtf(best), root = sqrtf(sigma);
    float ul = 0.f, vl = 0.f;  // lane l keeps element l of the winning columns
#pragma unroll
    for (int r = 0; r < MT; ++r) {
        const float a = __shfl(g[r], who), b = __shfl(v[r], who);
        if (c == r) {
            ul = a;
            vl = b;
        }
    }
    if (c < m) {
        Elem<T>::store(L + ((size_t)j * m + c) * m + k, sigma > 0.f ? ul / root : 0.f);
        Elem<T>::store(R + ((size_t)k * m + j) * m + c, vl * root);
    }
}

template <typename T>
void launch_t(const void* A, void* R, void* L, int m, hipStream_t st)
{
    const dim3 grid((unsigned)(m * m)), block(64);
    if (m <= 8) hipLaunchKernelGGL((project_kernel<T, 8>), grid, block, 0, st, (const T*)A, (T*)R, (T*)L, m);
    else if (m <= 16) hipLaunchKernelGGL((project_kernel<T, 16>), grid, block, 0, st, (const T*)A, (T*)R, (T*)L, m);
    else if (m <= 32) hipLaunchKernelGGL((project_kernel<T, 32>), grid, block, 0, st, (const T*)A, (T*)R, (T*)L, m);
    else hipLaunchKernelGGL((project_kernel<T, 64>), grid, block, 0, st, (const T*)A, (T*)R, (T*)L, m);
}

}  // namespace

bool project_supported(int m) { return m >= 1 && m <= 64; }

int launch_project(const void* A, void* R, void* L, int m, int dtype, hipStream_t st)
{
    if (!project_supported(m)) return -2;
    if (dtype == 0) launch_t<float>(A, R, L, m, st);
    else launch_t<bf16_t>(A, R, L, m, st);
    return hip_status(hipGetLastError());
}

}  // namespace monarch
