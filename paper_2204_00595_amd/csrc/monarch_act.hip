// Elementwise passes for the layers whose kernels do not apply the feed-forward block's nonlinearity
// in their own epilogues (monarch_fwd_bias_gelu, monarch_bwd_bias_gelu_in): one read and one write of
// the activation each.  The formulas are those of monarch_act.h.
#include "monarch_internal.h"
#include "monarch_device.h"
#include "monarch_act.h"

namespace monarch {

namespace {

// y (holding the pre-activation) -> y_pre (when wanted) and y = gelu(y); VEC elements per thread, 16 bytes
template <typename T, int VEC>
__global__ void __launch_bounds__(256) gelu_fwd_kernel(T* __restrict__ y, T* __restrict__ y_pre, size_t n)
{
    const size_t i0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (i0 >= n) return;
    if (i0 + VEC <= n) {
        typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
        const u32x4 raw = *reinterpret_cast<const u32x4*>(y + i0);
        if (y_pre) *reinterpret_cast<u32x4*>(y_pre + i0) = raw;
        alignas(16) T v[VEC];
        *reinterpret_cast<u32x4*>(v) = raw;
#pragma unroll
        for (int e = 0; e < VEC; ++e) Elem<T>::store(&v[e], gelu_f(Elem<T>::load(&v[e])));
        *reinterpret_cast<u32x4*>(y + i0) = *reinterpret_cast<u32x4*>(v);
    } else {
        for (size_t i = i0; i < n; ++i) {
            const T raw = y[i];
            if (y_pre) y_pre[i] = raw;
            Elem<T>::store(y + i, gelu_f(Elem<T>::load(&raw)));
        }
    }
}

// dx *= gelu'(x_pre)
template <typename T, int VEC>
__global__ void __launch_bounds__(256) gelu_bwd_kernel(T* __restrict__ dx, const T* __restrict__ x_pre, size_t n)
{
    const size_t i0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * VEC;
    if (i0 >= n) return;
    if (i0 + VEC <= n) {
        typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
        alignas(16) T g[VEC];
        alignas(16) T h[VEC];
        *reinterpret_cast<u32x4*>(g) = *reinterpret_cast<const u32x4*>(dx + i0);
        *reinterpret_cast<u32x4*>(h) = *reinterpret_cast<const u32x4*>(x_pre + i0);
#pragma unroll
        for (int e = 0; e < VEC; ++e) Elem<T>::store(&g[e], Elem<T>::load(&g[e]) * gelu_grad_f(Elem<T>::load(&h[e])));
        *reinterpret_cast<u32x4*>(dx + i0) = *reinterpret_cast<u32x4*>(g);
    } else {
        for (size_t i = i0; i < n; ++i) Elem<T>::store(dx + i, Elem<T>::load(dx + i) * gelu_grad_f(Elem<T>::load(x_pre + i)));
    }
}

template <int VEC>
bool grid_for(size_t n, unsigned* blocks)
{
    const size_t b = (n + (size_t)256 * VEC - 1) / ((size_t)256 * VEC);
    if (b > 0x7fffffffULL) return false;
    *blocks = (unsigned)b;
    return true;
}

}  // namespace

int launch_gelu_fwd(const Problem& pb, void* y, void* y_pre, hipStream_t st)
{
    const size_t n = (size_t)pb.B * pb.n_out();
    if (n == 0) return 0;
    unsigned blocks;
    if (pb.dtype == 0) {
        if (!grid_for<4>(n, &blocks)) return -2;
        hipLaunchKernelGGL((gelu_fwd_kernel<float, 4>), dim3(blocks), dim3(256), 0, st, (float*)y, (float*)y_pre, n);
    } else {
        if (!grid_for<8>(n, &blocks)) return -2;
        hipLaunchKernelGGL((gelu_fwd_kernel<bf16_t, 8>), dim3(blocks), dim3(256), 0, st, (bf16_t*)y, (bf16_t*)y_pre, n);
    }
    return hip_status(hipGetLastError());
}

int launch_gelu_bwd(const Problem& pb, void* dx, const void* x_pre, hipStream_t st)
{
    const size_t n = (size_t)pb.B * pb.n_in;
    if (n == 0) return 0;
    unsigned blocks;
    if (pb.dtype == 0) {
        if (!grid_for<4>(n, &blocks)) return -2;
        hipLaunchKernelGGL((gelu_bwd_kernel<float, 4>), dim3(blocks), dim3(256), 0, st, (float*)dx, (const float*)x_pre, n);
    } else {
        if (!grid_for<8>(n, &blocks)) return -2;
        hipLaunchKernelGGL((gelu_bwd_kernel<bf16_t, 8>), dim3(blocks), dim3(256), 0, st, (bf16_t*)dx, (const bf16_t*)x_pre, n);
    }
    return hip_status(hipGetLastError());
}

}  // namespace monarch
